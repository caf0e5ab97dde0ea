/*
 * ellm.h — C ABI of libellm: chunk-backed virtual KV tensors, KV append and batched GQA decode
 * attention for AMD MI355X (gfx950).
 *
 * The operations follow the eLLM paper (arXiv 2506.15155):
 *   - a unified physical pool of fixed-size chunks shared by the KV cache and activations
 *     (Introduction "Our solution"; Sec. 2.1 "Virtual Tensor Abstraction");
 *   - a KV virtual tensor ("KV eTensor") per request that reserves its whole token range up
 *     front, is logically contiguous, and gets physical chunks mapped on demand at write time;
 *     its slots are aligned to the chunk granularity (Sec. 2.1.1 "Virtualization Design");
 *   - inflation / deflation: ownership of idle chunks moves between the activation side and the
 *     KV side of the pool and the chunks are remapped into KV tensors (Sec. 2.2.1);
 *   - offloading / fetching: the KV chunks of a request are moved to CPU DRAM and brought back
 *     before the request decodes again (Sec. 2.2.2);
 *   - decode: every sequence writes one new token per iteration (Sec. 3.1) and attends over its
 *     whole cached context with standard softmax attention, grouped-query or multi-head
 *     (Sec. 4.1 "Models"; Sec. 5 "Efficient Kernels").
 *
 * The paper maps chunks with the GPU driver's virtual-memory API. By default this library keeps
 * the virtual-to-physical map in software instead: one int32 table row per tensor, token t living
 * in slot t / T_c at row t % T_c of the chunk the table names, read directly by the kernels. A
 * pool created with ELLM_POOL_DRIVER_MAPPED does it the paper's way as well: the driver maps the
 * chunks into each tensor's address range and the kernels read contiguous addresses.
 *
 * All pointers say "host" or "device" below. No call allocates memory the caller has to free
 * except ellm_pool_create (freed by ellm_pool_destroy). A pool is NOT thread-safe: one host
 * thread drives it. Every call validates its whole argument set on the host before it changes any
 * state or launches anything; a call that returns an error from these checks has changed nothing.
 * The one error that can come later is ELLM_ERR_HIP from a kernel launch the runtime refuses: a
 * call that works in several launches (more than 128 requests) has then done the work of the
 * launches before it, completely, and nothing of the rest (see ellm_kv_append).
 *
 * Device memory of the library: the mirror of the chunk tables and the workspace for partial
 * attention results, both allocated once by the first call that needs the device (or by
 * ellm_pool_prepare) and freed by ellm_pool_destroy; ellm_workspace_bytes tells the size of the
 * second. After that first call ellm_kv_append, ellm_decode_attention and ellm_kv_append_decode
 * neither allocate nor wait for the device.
 */
#ifndef ELLM_H
#define ELLM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- return codes (0 = success, negative = error) ------------------------------------------ */
#define ELLM_OK                 0
#define ELLM_ERR_INVALID       (-1)  /* malformed argument, bad handle, duplicate id, slot in use  */
#define ELLM_ERR_OOM           (-2)  /* no free device chunk (even after allowed inflation), or no
                                        free tensor handle                                          */
#define ELLM_ERR_OWNED         (-3)  /* chunk is mapped, busy, or belongs to the other owner       */
#define ELLM_ERR_UNMAPPED      (-4)  /* operation touches a slot that has no chunk                 */
#define ELLM_ERR_NOT_RESIDENT  (-5)  /* operation touches a slot whose chunk is in host memory     */
#define ELLM_ERR_RANGE         (-6)  /* slot / token / chunk index outside its range               */
#define ELLM_ERR_EMPTY         (-7)  /* decode over a tensor that holds no token                   */
#define ELLM_ERR_HOST_FULL     (-8)  /* not enough free host slots for an offload                  */
#define ELLM_ERR_HIP           (-9)  /* a HIP runtime call failed (text in ellm_last_error)        */
#define ELLM_ERR_NO_DEVICE     (-10) /* compute call on a pool created with ELLM_POOL_METADATA_ONLY */

/* ---- constants ------------------------------------------------------------------------------ */
#define ELLM_OWNER_KV    0   /* chunk belongs to the KV side of the pool          */
#define ELLM_OWNER_ACT   1   /* chunk belongs to the activation side of the pool  */

#define ELLM_CHUNK_FREE   0  /* idle, may be mapped (KV side) or transferred      */
#define ELLM_CHUNK_MAPPED 1  /* backs exactly one (tensor, slot)                  */
#define ELLM_CHUNK_BUSY   2  /* holds live activations; KV side may not touch it  */

#define ELLM_BF16 1          /* the only element type: bfloat16, 2 bytes          */

#define ELLM_MAP_ALLOW_INFLATE 1u  /* map may take FREE activation-owned chunks (Sec. 2.2.1)  */

#define ELLM_POOL_METADATA_ONLY 1u /* pool flag: no device behind the pool. Host state machine
                                      only: append advances lengths without launching, offload and
                                      fetch move bookkeeping without copying bytes, decode returns
                                      ELLM_ERR_NO_DEVICE after validating. For host-logic tests.  */

#define ELLM_POOL_DRIVER_MAPPED 2u  /* pool flag: the paper's own mechanism (Sec. 2.1.1 "Virtualization
                                      Design", Sec. 3.2). The library creates every chunk as a physical
                                      allocation of its own (device_base must be NULL, device_bytes says how
                                      many; chunk_bytes must be a multiple of the driver's allocation
                                      granularity). A tensor is a reserved virtual address range; a chunk that
                                      backs one of its slots is mapped there by the driver's virtual-memory
                                      calls, and the append and attention kernels read the tensor as
                                      contiguous addresses, with no table. The host table is kept all the
                                      same (it is what every check and every introspection call reads), and
                                      all chunks are mapped a second time, in id order, into one range
                                      (ellm_pool_get_device_base), through which copies address them. A call
                                      that changes table entries does not make the driver calls itself: it
                                      hands them, in order, to a thread the pool owns (Sec. 3.1: chunks are
                                      mapped ahead of their first use and unmapping is kept off the critical
                                      path), and returns. A compute call waits, on the host, until the slots
                                      it is about to touch have been mapped; a slot mapped a step ahead
                                      (ellm_pool_premap_next) is ready by then. A chunk taken out of a slot
                                      (unmap, offload, destroy, chunks taken back by acquire) is unmapped by
                                      that thread once the kernels enqueued so far have finished. A driver
                                      error met by the thread is returned, as ELLM_ERR_HIP, by the next call
                                      that waits for it and by every such call after that. ellm_pool_sync
                                      also waits for the thread. Same results, bit for bit, as a pool
                                      without the flag. */

/* Table-entry encoding (compared bit-exactly by tests):
 *   e >= 0   device chunk id
 *   e == -1  slot has no chunk
 *   e <= -2  chunk content is in host slot (-e - 2)                                            */
#define ELLM_ENTRY_UNMAPPED (-1)
#define ELLM_ENTRY_FROM_HOST_SLOT(s) (-(int32_t)(s) - 2)
#define ELLM_ENTRY_TO_HOST_SLOT(e)   (-(int32_t)(e) - 2)

typedef struct ellm_pool ellm_pool;   /* opaque, owned by the library */
typedef int32_t ellm_tensor_id;       /* dense handle >= 0            */

/*
 * Pool geometry.
 *   bpt  = bytes per token of one layer = 2 (K and V) * n_kv_heads * head_dim * 2 bytes
 *   T_c  = tokens per chunk             = floor(chunk_bytes / bpt)        (must be >= 1)
 *   n_chunks     = floor(device_bytes / chunk_bytes)
 *   n_host_slots = floor(host_bytes   / chunk_bytes)                      (may be 0)
 *
 * Layout of one chunk (the migrated bytes and every reader depend on it): element
 * (kv head h, plane p (0 = K, 1 = V), token row r < T_c, dim d) sits at byte offset
 *   ((h * 2 + p) * T_c + r) * head_dim * 2 + d * 2.
 * Bytes past 2 * n_kv_heads * T_c * head_dim * 2 are slack: never read by attention, but copied
 * by offload / fetch, which always move whole chunks.
 */
typedef struct ellm_pool_desc {
  void*    device_base;      /* device, caller-owned, 256-byte aligned; NULL with METADATA_ONLY and
                                DRIVER_MAPPED                                                       */
  uint64_t device_bytes;
  void*    host_base;        /* host, caller-owned, pinned; NULL iff host_bytes < chunk_bytes     */
  uint64_t host_bytes;
  uint32_t chunk_bytes;      /* multiple of 256                                                   */
  uint16_t n_q_heads;
  uint16_t n_kv_heads;       /* n_q_heads % n_kv_heads == 0; group size G = n_q / n_kv <= 64      */
  uint16_t head_dim;         /* 64 or 128                                                         */
  uint16_t dtype;            /* ELLM_BF16                                                         */
  uint32_t max_tensors;      /* tensor handles 0 .. max_tensors-1                                 */
  uint32_t max_slots_per_tensor;
  uint32_t flags;            /* 0, ELLM_POOL_METADATA_ONLY or ELLM_POOL_DRIVER_MAPPED             */
  uint32_t reserved;         /* must be 0                                                         */
  const uint8_t* initial_owner; /* host, n_chunks bytes of ELLM_OWNER_*; NULL = all KV.
                                   Every chunk starts FREE.                                       */
} ellm_pool_desc;

/* Create a pool over caller-owned buffers (Sec. 2.1: one unified physical pool).
 * Errors: INVALID for any violated constraint above. No HIP call is made here; device-side
 * metadata is created lazily by the first call that launches or copies. A driver-mapped pool is
 * the exception: its chunks are created and mapped here (errors: HIP, and INVALID for a chunk size
 * the driver's granularity does not divide). */
int ellm_pool_create(const ellm_pool_desc* desc, ellm_pool** out);

/* Drains the library's streams, frees its metadata. Caller buffers are untouched. */
int ellm_pool_destroy(ellm_pool* pool);

/* Bytes of device workspace a pool of this geometry allocates for the partial results of split
 * decode attention (Sec. 5 "Efficient Kernels": the sequence is split and partial softmax results
 * are combined), for batches of up to max_batch requests: a decode launch covers at most 128
 * requests and runs one wave per SIMD of the GPU; every wave writes at most one partial result per
 * request its share touches, so a launch needs at most SIMDs + n_kv_heads * (min(max_batch, 128) - 1)
 * partial slots of G * (head_dim + 2) floats, and the launches of one call reuse the same slots.
 * Uses the current HIP device's SIMD count (a nominal 1024 without a device). Only the head
 * counts and head_dim of desc are read. 0 for a bad argument. */
uint64_t ellm_workspace_bytes(const ellm_pool_desc* desc, int32_t max_batch);

/* Create the device-side metadata now (table mirror, workspace, side streams, events) and bring
 * the table mirror up to date on `stream`, instead of leaving it to the first append / decode /
 * migration call. The only call besides that first one that allocates device memory. No-op on a
 * metadata-only pool. Errors: HIP. */
int ellm_pool_prepare(ellm_pool* pool, void* stream);

/* Reserve a virtual tensor of max_tokens tokens (Sec. 2.1.1: virtual range = maximum context,
 * no physical chunk yet). n_slots = ceil(max_tokens / T_c). Returns the lowest unused handle.
 * Errors: INVALID (max_tokens < 1), RANGE (n_slots > max_slots_per_tensor), OOM (no handle). */
int ellm_tensor_create(ellm_pool* pool, int64_t max_tokens, ellm_tensor_id* out);

/* Release a tensor: its device chunks become FREE (owner unchanged), its host slots are freed,
 * the handle becomes reusable. Errors: INVALID (bad handle). */
int ellm_tensor_destroy(ellm_pool* pool, ellm_tensor_id id);

/* Map chunks into slots [first_slot, first_slot + n_slots) (Sec. 2.1.1 on-demand allocation;
 * Sec. 2.2.1 steps 1, 3, 4 when ELLM_MAP_ALLOW_INFLATE is set).
 *   chunk_ids (host): n_slots explicit ids, slot first_slot + i gets chunk_ids[i]; or NULL, then
 *   the pool takes the lowest-numbered FREE KV-owned chunks in ascending order and, only if those
 *   run out and ALLOW_INFLATE is set, the lowest-numbered FREE ACT-owned chunks, whose owner
 *   becomes KV.
 * Checks, in this order: bad handle or n_slots < 0 -> INVALID; n_slots == 0 -> OK; slot range ->
 * RANGE; any target slot not empty -> INVALID; explicit ids in order: id outside the pool -> RANGE,
 * not FREE -> OWNED, repeated -> OWNED, ACT-owned without ALLOW_INFLATE -> OWNED; pool-chosen:
 * too few chunks -> OOM. */
int ellm_tensor_map_chunks(ellm_pool* pool, ellm_tensor_id id, int32_t first_slot, int32_t n_slots,
                           const int32_t* chunk_ids, uint32_t flags);

/* Undo a mapping of slots that hold no live token (slot index >= ceil(len / T_c)), e.g. a
 * speculative pre-map (Sec. 3.1). Chunks become FREE, host slots are released.
 * Checks: bad handle or n_slots < 0 -> INVALID; range -> RANGE; a slot below ceil(len / T_c)
 * -> INVALID; an empty slot -> UNMAPPED. */
int ellm_tensor_unmap_chunks(ellm_pool* pool, ellm_tensor_id id, int32_t first_slot, int32_t n_slots);

/* ---- request turnover (Sec. 2.1.2 "Memory Management Strategy"; Sec. 3.1 pre-mapping) --------- */

/* The request is over (Sec. 2.1.2): the tensor is not unmapped but becomes "mapped and available".
 * Its length drops to 0; its leading run of slots that have a device chunk stays mapped (that run,
 * times T_c, is its mapped size); whatever lies behind the first slot without a device chunk (host
 * copies, stray mappings) is given back. A released tensor takes no call except
 * ellm_tensor_acquire (as a candidate), ellm_tensor_destroy, ellm_tensor_get_table and
 * ellm_tensor_is_released; every other call on it -> INVALID.
 * Checks: bad or already released handle -> INVALID. */
int ellm_tensor_release(ellm_pool* pool, ellm_tensor_id id);

/* A new request that needs room for need_tokens now and max_tokens at most. Best fit (the arg min
 * of Sec. 2.1.2): of the released tensors whose max_tokens is at least the one asked for and whose
 * mapped size is at least need_tokens, the one with the smallest mapped size; equal sizes: the
 * lowest handle. It becomes live again with length 0 and its own max_tokens; no mapping changes,
 * nothing to do on the device. Without such a tensor, on-demand mapping: a fresh tensor (lowest
 * free handle) gets ceil(need_tokens / T_c) chunks in slots 0.., taken in this order: FREE KV
 * chunks ascending; then chunks taken back from released tensors (smallest mapped size first,
 * equal sizes lowest handle first, each from its last mapped slot downwards); then, with
 * ELLM_MAP_ALLOW_INFLATE, FREE ACT chunks ascending. All or nothing.
 * Checks: need_tokens < 0, max_tokens < 1, need_tokens > max_tokens, unknown flag -> INVALID;
 * max_tokens needs more than max_slots_per_tensor slots -> RANGE; on-demand: no free handle, or
 * too few chunks -> OOM. */
int ellm_tensor_acquire(ellm_pool* pool, int64_t need_tokens, int64_t max_tokens, uint32_t flags,
                        ellm_tensor_id* out);

/* 1 if the tensor is released, 0 if it is live; bad handle -> INVALID. */
int ellm_tensor_is_released(ellm_pool* pool, ellm_tensor_id id);

/* Speculative pre-mapping (Sec. 3.1): every sequence is assumed to produce one more token, so each
 * listed tensor whose next token would open a slot that has no chunk (len < max_tokens,
 * len % T_c == 0, slot len / T_c empty) gets one mapped now, pool-chosen as in
 * ellm_tensor_map_chunks, in batch order. All or nothing; *n_mapped (may be NULL) = chunks mapped.
 * Checks: batch < 0, bad / released / repeated handle, unknown flag -> INVALID; too few chunks -> OOM. */
int ellm_kv_premap_next(ellm_pool* pool, const ellm_tensor_id* ids, int32_t batch, uint32_t flags,
                        int32_t* n_mapped);

/* The same with a longer view (Sec. 3.1 maps "ahead of time"; how far is the caller's policy): every
 * listed tensor is assumed to produce tokens_ahead more tokens, as far as its max_tokens allows, and
 * every slot those tokens would be written to that has no chunk gets one now, in batch order and,
 * within a tensor, in slot order; slots that hold a host copy are left alone. tokens_ahead == 1 is
 * ellm_kv_premap_next. In a driver-mapped pool this is what gives the pool's mapper thread the time
 * to make the driver calls before the slot's first write. All or nothing; *n_mapped (may be NULL) =
 * chunks mapped.
 * Checks: as ellm_kv_premap_next, and tokens_ahead < 1 -> INVALID. */
int ellm_kv_premap_ahead(ellm_pool* pool, const ellm_tensor_id* ids, int32_t batch, int64_t tokens_ahead,
                         uint32_t flags, int32_t* n_mapped);

/* Push the table changes made so far to the device mirror now, ordered on `stream`, instead of at
 * the start of the next append / decode call: with ellm_kv_premap_next this moves the mapping
 * work of the next step out of its way (Sec. 3.1). The changed entries travel in the arguments of
 * small kernels (448 per launch); the call does not wait for the device. No-op on a metadata-only
 * pool. */
int ellm_pool_flush_tables(ellm_pool* pool, void* stream);

/* Ownership transfer of FREE chunks between the two sides of the pool (Sec. 2.2.1 step 3 for
 * new_owner = KV, "deflation" for new_owner = ACT). A chunk that already has new_owner is left
 * as it is. Checks: n < 0 or bad owner -> INVALID; per id in order: outside pool -> RANGE,
 * not FREE -> OWNED, repeated -> INVALID.
 * A chunk that an offload has just freed may still be read by its copy, and one whose tensor was
 * destroyed right after a fetch may still be written: with new_owner = ACT the call returns only
 * when the library's copies through the listed chunks have finished (the host waits), so whoever
 * fills them next cannot race with a copy. Kernels of append / decode calls that still read a
 * chunk are the caller's to order: they run on the caller's stream. */
int ellm_pool_transfer(ellm_pool* pool, const int32_t* chunk_ids, int32_t n, int new_owner);

/* Stand-in for live activation tensors (the paper's activation allocator and its garbage
 * collection, Sec. 2.2.1 step 2, are outside this library): mark ACT-owned chunks BUSY (busy = 1,
 * they must be FREE) or FREE again (busy = 0, they must be BUSY).
 * Checks per id in order: outside pool -> RANGE, not ACT-owned -> OWNED, wrong state -> OWNED for
 * busy = 1 / INVALID for busy = 0, repeated -> INVALID.
 * busy = 1 waits for the library's copies through the listed chunks like ellm_pool_transfer. */
int ellm_pool_set_act_busy(ellm_pool* pool, const int32_t* chunk_ids, int32_t n, int busy);

/* Append new tokens to a batch of tensors (Sec. 3.1: one token per sequence per decode iteration;
 * n_new > 1 is the prefill-side write).
 *   ids (host): batch distinct handles. n_new (host): tokens per request, NULL = 1 each.
 *   k_new, v_new (device): [sum(n_new)][n_kv_heads][head_dim] bf16, request b's tokens start at row
 *   sum(n_new[0..b)). Token i of request b is written at position len_b + i; afterwards
 *   len_b += n_new[b]. Enqueued on `stream` (a hipStream_t); returns without waiting.
 * Checks: batch < 0 -> INVALID; per request in order: bad or repeated handle, n_new < 0 -> INVALID;
 * len + n_new > max_tokens -> RANGE; slots covering the new tokens in ascending order: empty ->
 * UNMAPPED, on host -> NOT_RESIDENT. NULL k_new / v_new with tokens to write -> INVALID.
 * More than 128 requests are written by one launch per 128; the lengths of a group advance when
 * its launch has been accepted. If the runtime refuses a launch (HIP), the groups before it have
 * been appended completely, rows and lengths, and the refused group and those after it not at all. */
int ellm_kv_append(ellm_pool* pool, const ellm_tensor_id* ids, int32_t batch, const int32_t* n_new,
                   const void* k_new, const void* v_new, void* stream);

/* Batched decode attention: one query token per request over its whole cached context.
 *   q (device): [batch][n_q_heads][head_dim] bf16; out (device): same shape, bf16.
 *   For q head h, kv head g = h / G:  s_t = scale * <q_h, K_t,g>,  w = softmax_t(s),
 *   out_h = sum_t w_t * V_t,g  for t = 0 .. len-1, no mask. scale = 0 selects 1/sqrt(head_dim).
 *   fp32 accumulation (softmax weights are rounded to bf16 before they multiply V and before they
 *   are summed), output rounded to nearest-even bf16. Split over the sequence with a partition
 *   that depends only on the lengths in the batch, the pool geometry and the device's wave
 *   capacity, never on physical chunk ids, so results are bitwise reproducible and invariant
 *   under remapping.
 * Checks: batch < 0, NULL q / out, non-finite scale -> INVALID; per request in order: bad handle ->
 * INVALID, len == 0 -> EMPTY; slots 0 .. ceil(len / T_c) - 1 ascending: empty -> UNMAPPED, on host
 * -> NOT_RESIDENT. Enqueued on `stream`; returns without waiting. */
int ellm_decode_attention(ellm_pool* pool, const ellm_tensor_id* ids, int32_t batch, const void* q,
                          void* out, float scale, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid it): ellm_decode_attention with the partial results kept in a fixed
 * workspace of ELLM_NOALLOC_WORKSPACE_BYTES that is part of the library's own device image instead
 * of the pool's allocated one. The call allocates and frees nothing on the device and never waits
 * for it. Same arguments, checks, kernels, partition and output bits as ellm_decode_attention.
 * Additional errors: INVALID if the pool's device-side metadata has not been created yet (creating
 * it allocates; ellm_pool_prepare and every append / migration call do it, so a pool whose tensors
 * hold tokens has it); RANGE if a launch of the batch needs more partial results than the fixed workspace holds (a
 * launch of n requests needs at most SIMDs + n_kv_heads * (n - 1) slots of G * (head_dim + 2) * 4
 * bytes: 3.2 MB for 64 requests of 32 q / 8 kv heads of 128 on 1024 SIMDs). Every GPU the library
 * runs on holds one such workspace from load to process end, shared by all pools and all calls of
 * this entry point on that GPU: calls that overlap in time on one GPU (two streams, two pools)
 * race on it and must be ordered by the caller. Nothing in it needs clearing between calls: every
 * slot a call reads, the same call has written before. */
#define ELLM_NOALLOC_WORKSPACE_BYTES (16u << 20)
int ellm_decode_attention_noalloc(ellm_pool* pool, const ellm_tensor_id* ids, int32_t batch, const void* q,
                                  void* out, float scale, void* stream);

/* One decode iteration in a single pass (Sec. 3.1: every sequence writes one token, then attends
 * over its whole context): the same tables, lengths, chunk bytes and output bits as
 * ellm_kv_append(pool, ids, batch, NULL, k_new, v_new, stream) followed by
 * ellm_decode_attention(pool, ids, batch, q, out, scale, stream), but the new K/V rows are taken
 * from k_new / v_new by the attention kernel itself, which also writes them into their chunks, so
 * no separate append kernel runs.
 *   k_new, v_new (device): [batch][n_kv_heads][head_dim] bf16; q, out (device): [batch][n_q_heads][head_dim].
 * Checks: batch < 0, NULL q / out, non-finite scale -> INVALID; then the checks of ellm_kv_append
 * with one token per request; NULL k_new / v_new with batch > 0 -> INVALID; then the checks of
 * ellm_decode_attention on the lengths after the append. A call that fails these checks has changed
 * nothing; a refused launch (HIP) leaves the groups of 128 requests before it appended and decoded
 * and the rest untouched, as in ellm_kv_append. */
int ellm_kv_append_decode(ellm_pool* pool, const ellm_tensor_id* ids, int32_t batch, const void* k_new,
                          const void* v_new, const void* q, void* out, float scale, void* stream);

/* Offload (Sec. 2.2.2): copy the chunks of slots [first_slot, first_slot + n_slots) to host
 * slots (lowest free host slot first, slots in ascending order), free the device chunks (owner
 * stays KV), entry := host code. The copies run on a side stream of the library (offloads and
 * fetches have one each, so the two directions overlap). Ordering is kept per chunk and per host
 * slot: a copy waits for the append / decode calls already enqueued that touch its chunks (not
 * for others: a copy for one tensor runs under the attention of another), and for earlier copies
 * in the other direction through the same chunk or host slot; a later append / decode call waits,
 * on its own stream, for the copies that touched its tensors' chunks. The append / decode calls
 * of a pool form one sequence: a call on another stream than the call before it is first made to
 * wait, on its stream, for everything that call enqueued.
 * Checks: bad handle, n_slots < 0 -> INVALID; range -> RANGE; slots ascending: empty -> UNMAPPED,
 * already on host -> NOT_RESIDENT; fewer than n_slots free host slots, or more occupied host slots
 * than the logical host buffer allows -> HOST_FULL. */
int ellm_chunk_deflate_to_host(ellm_pool* pool, ellm_tensor_id id, int32_t first_slot, int32_t n_slots);

/* Fetch (Sec. 2.2.2): bring host-resident slots back into FREE KV-owned device chunks
 * (explicit ids, or NULL = lowest-numbered first; never takes ACT-owned chunks — transfer them
 * first), release the host slots, entry := new chunk id. Same ordering rules as offload.
 * Checks: bad handle, n_slots < 0 -> INVALID; range -> RANGE; slots ascending: empty -> UNMAPPED,
 * already on device -> INVALID; explicit ids in order: outside pool -> RANGE, not FREE / repeated /
 * ACT-owned -> OWNED; pool-chosen: too few -> OOM. */
int ellm_chunk_inflate_from_host(ellm_pool* pool, ellm_tensor_id id, int32_t first_slot, int32_t n_slots,
                                 const int32_t* chunk_ids);

/* Logical host buffer (Sec. 2.3.2): the part of the host slots that offloads may fill. Offloads
 * fail with HOST_FULL once occupied host slots + the request would exceed it; shrinking it evicts
 * nothing that is already stored. Initially all host slots. n outside 0 .. host slots -> RANGE. */
int ellm_pool_set_logical_host_slots(ellm_pool* pool, int32_t n);
int ellm_pool_get_logical_host_slots(ellm_pool* pool, int32_t* n);

/* SLO-aware scaling of the logical host buffer (Sec. 2.3.2). configure: the two thresholds (same
 * unit as the latencies passed to observe), the tuning factor alpha (paper: 2), the window in
 * scheduling iterations (paper: 5) and the violations within it that make an event (paper: 3).
 * observe: the latencies of one scheduling iteration, time to first token and time per output
 * token (a negative value = none measured). The paper fixes: an event when the latency exceeded
 * its threshold `threshold` times within the window; time per output token -> the buffer shrinks,
 * time to first token -> it grows, at a rate set by alpha. This library's reading of what it
 * leaves open: shrink to floor(size / alpha), grow to min(all host slots, ceil(max(1, size) *
 * alpha)); when both events fall together the buffer shrinks; the window slides over the
 * iterations since the last change and starts empty after one. *logical_host_slots (may be NULL)
 * receives the size after the call.
 * Checks: thresholds <= 0, alpha <= 1, window < 1, threshold outside 1 .. window, NaN latency,
 * observe before configure -> INVALID. */
int ellm_pool_slo_configure(ellm_pool* pool, double ttft_slo, double tpot_slo, double alpha, int32_t window,
                            int32_t threshold);
int ellm_pool_slo_observe(ellm_pool* pool, double ttft, double tpot, int32_t* logical_host_slots);

/* Block until all migrations enqueued so far have finished (and, in a driver-mapped pool, all
 * mappings asked for have been made). Returns HIP on an asynchronous fault. */
int ellm_pool_sync(ellm_pool* pool);

/* ---- introspection (host state, for bit-exact checks) -------------------------------------- */
/* Address of chunk 0 (chunk c is at base + c * chunk_bytes): the caller's device_base, or for a
 * driver-mapped pool the range into which the library has mapped all its chunks. */
int ellm_pool_get_device_base(ellm_pool* pool, void** base);
/* Driver-mapped pools: how many chunk mappings the driver has made and removed for this pool's
 * tensors so far and the host microseconds spent in those calls (map + set-access, unmap), the
 * figure the paper reports as the share of time in virtual-memory operations (Sec. 4.6). Any out
 * pointer may be NULL; zeros for other pools. */
int ellm_pool_get_mapping_stats(ellm_pool* pool, int64_t* n_map, double* us_map, int64_t* n_unmap, double* us_unmap);
/* Host microseconds the pool's callers have spent waiting for the thread that makes the driver calls
 * (host): what is left of the figure above on the critical path. */
int ellm_pool_get_mapping_wait(ellm_pool* pool, double* us_waited);
/* Geometry: any out pointer may be NULL. */
int ellm_pool_get_geometry(ellm_pool* pool, int32_t* n_chunks, int32_t* tokens_per_chunk,
                           int32_t* n_host_slots, uint64_t* bytes_per_token);
/* Copies min(cap, n_slots) table entries to out (host); n_slots / len may be NULL. */
int ellm_tensor_get_table(ellm_pool* pool, ellm_tensor_id id, int32_t* out, int32_t cap,
                          int32_t* n_slots, int64_t* len);
/* Per chunk (host arrays of n_chunks, any may be NULL): owner, state, and for MAPPED chunks the
 * (tensor, slot) they back, else -1. */
int ellm_pool_get_owner_state(ellm_pool* pool, uint8_t* owner, uint8_t* state,
                              int32_t* mapped_tensor, int32_t* mapped_slot);
/* Per host slot (host arrays of n_host_slots, any may be NULL): the (tensor, slot) stored, else -1. */
int ellm_pool_get_host_slots(ellm_pool* pool, int32_t* tensor, int32_t* slot);
/* The partition the next decode over these handles would use: n_split[b] (host array of batch) is
 * the number of partial results of each (request b, kv head) pair, i.e. the number of waves whose
 * share of the kv head's tiles holds tiles of the request; *split_tokens is the largest share, in
 * tokens (a multiple of 64). For tests of the partition. */
int ellm_decode_plan(ellm_pool* pool, const ellm_tensor_id* ids, int32_t batch,
                     int32_t* n_split, int32_t* split_tokens);
/* Override the tokens per wave (rounded down to whole 64-token tiles, at least one; 0 = automatic:
 * one wave per SIMD of the GPU). For tests that compare partitions. While an override (this one or
 * ellm_debug_set_waves) is in force, a decode call whose partition needs more partial results than
 * the workspace holds replaces the workspace, which waits for the device; without an override that
 * cannot happen. */
int ellm_pool_set_split_tokens(ellm_pool* pool, int32_t split_tokens);

/* Measurement hooks. profile_enable(max_records > 0) makes each decode launch attach a pair of
 * HIP events to its partial-pass kernel (the kernel that streams K/V) on the caller's stream, which
 * take that kernel's own start and end times (the runtime's extended launch: no marker of its own
 * goes into the stream), for up to max_records launches; max_records = 0 switches it off. profile_collect waits for the
 * recorded launches, writes their durations in milliseconds to ms (host, cap entries), stores the
 * number recorded in *n and starts over. Not part of the paper's method. */
int ellm_pool_profile_enable(ellm_pool* pool, int32_t max_records);
/* Time only every stride-th decode launch (default 1 = all): an event pair costs a few microseconds
 * of stream time, which a throughput measurement should not pay on every launch. */
int ellm_pool_profile_stride(ellm_pool* pool, int32_t stride);
int ellm_pool_profile_collect(ellm_pool* pool, float* ms, int32_t cap, int32_t* n);

/* Calibration kernels for measurement; none computes anything of the method.
 *   debug_copy: dst[0..bytes) = src[0..bytes) (device, bytes % 16 == 0): the known-size kernel that
 *     hardware byte counters are scaled against.
 *   debug_stream_read: reads src[0..bytes) (device) and discards it: the read ceiling of the GPU.
 *     sink: device, 4 bytes.
 *   debug_kv_stream_read: reads exactly the K/V rows a decode over `ids` would read, with the same
 *     work partition and load shape, and discards them: the ceiling of the access pattern.
 *     Same checks as ellm_decode_attention. */
int ellm_debug_copy(void* dst, const void* src, uint64_t bytes, void* stream);
int ellm_debug_stream_read(const void* src, uint64_t bytes, void* sink, void* stream);
int ellm_debug_kv_stream_read(ellm_pool* pool, const ellm_tensor_id* ids, int32_t batch, void* sink, void* stream);

/* Waves of a decode launch as a percentage (1..1600, default 100) of the library's choice, one
 * wave per SIMD of the GPU; for measurements of the work partition. Results do not depend on it
 * beyond rounding order. */
int ellm_debug_set_waves(ellm_pool* pool, int32_t percent);

/* Measurement only: what the paper's own mechanism costs on this GPU (Sec. 2.1.1, Sec. 3.2: chunks
 * mapped into a reserved virtual range through the driver's virtual-memory calls). Creates
 * n_chunks (1..4096) physical allocations of chunk_bytes (rounded up to the driver's granularity),
 * maps each into one reserved range and makes it accessible, clears the range, unmaps and releases
 * everything. us (host, 4 doubles) receives host microseconds per chunk for: create, map +
 * set-access, unmap, release. HIP when the driver refuses a call (text in ellm_last_error). */
int ellm_debug_vmm_latency(uint64_t chunk_bytes, int32_t n_chunks, double* us);
/* A device buffer of n_chunks pieces of chunk_bytes (a multiple of the driver's allocation
 * granularity, 2 MiB here), each piece a physical allocation of its own, mapped into one reserved
 * virtual range in an order shuffled by seed and filled with the 16-bit pattern fill16: the
 * memory a pool sits in under the paper's mechanism, for bandwidth comparisons against one plain
 * allocation (pass *base as ellm_pool_desc.device_base). The library owns the buffer until
 * ellm_debug_vmm_buffer_destroy(base), which the caller invokes after destroying every pool in it.
 * Errors: INVALID (arguments, unknown base), HIP. */
int ellm_debug_vmm_buffer_create(uint64_t chunk_bytes, int32_t n_chunks, uint32_t seed, uint16_t fill16,
                                 void** base, uint64_t* bytes);
int ellm_debug_vmm_buffer_destroy(void* base);

/* Driver-mapped pools, for comparisons in one pool: on != 0 makes append and attention read the
 * chunks through the software table (in the range of ellm_pool_get_device_base) as in a plain pool;
 * 0 goes back to the tensors' own address ranges. Same output bits. INVALID for other pools. */
int ellm_debug_set_table_kernels(ellm_pool* pool, int on);
/* Driver-mapped pools, for measurements: on == 0 makes every call that changes table entries wait
 * until the driver calls it asked for have been made (what the pool would cost without its mapper
 * thread); != 0 (the default) goes back to handing them over. INVALID for other pools. */
int ellm_debug_set_async_mapping(ellm_pool* pool, int on);
/* Offload and fetch move their chunks with the runtime's copy calls (copy engines, beside the
 * kernels). on != 0 makes them use the library's copy kernel instead (one launch per call, the GPU
 * reading or writing the pinned host buffer directly) where the GPU can address the host buffer:
 * faster when nothing else runs, but it takes compute units from the kernels beside it. 0 (the
 * default) goes back. For measurements; same bytes either way. */
int ellm_debug_set_copy_kernels(ellm_pool* pool, int on);
/* Test hook for the error path of a driver-mapped pool's mapper thread: the nth mapping it is asked
 * for from now on (1 = the next one; 0 = none) is not made and counts as refused by the driver. Every
 * later call that would launch a kernel on the pool, or that waits for the thread, then returns
 * ELLM_ERR_HIP and launches nothing; ellm_pool_destroy still works. INVALID for other pools. */
int ellm_debug_fail_mapping(ellm_pool* pool, int32_t nth);

/* Test hook for the error path of calls that work in several launches: the nth kernel launch of
 * ellm_kv_append / ellm_decode_attention / ellm_kv_append_decode from now on (1 = the next one) is
 * refused as if the runtime had returned an error: nothing is launched, the call returns HIP. Also
 * on metadata-only pools, where it applies to the launches a device pool would make. 0 = off. */
int ellm_debug_fail_launch(ellm_pool* pool, int32_t nth);

/* O(n) consistency scan of the host state (tables, chunk records, free lists, host slots agree;
 * no chunk backs two slots). Returns 0 when consistent, else a positive rule number. */
int ellm_pool_self_check(ellm_pool* pool);

/* Text of the last error raised on this thread (never NULL). */
const char* ellm_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ELLM_H */
