// HIP kernels for gfx950 (MI355X): table patch, KV append, split-K decode attention, combine.
//
// Decode attention is a streaming read of every cached K and V row once per step (the paper calls
// auto-regressive generation memory-bound, Introduction and Sec. 2.2.1), so the kernels are built
// around 128-bit coalesced loads from the scattered chunks and keep all arithmetic on ordinary
// vector lanes; there is no dense contraction here that would pay for the matrix cores.
//
// Per-launch metadata (which tensors, their lengths, where each request's work items start) is
// passed by value in the kernel arguments, so a launch needs no host-to-device copy and no staging
// buffer whose lifetime would have to be tracked. The chunk tables live in a device mirror that is
// patched, also through kernel arguments, whenever the host changes an entry.
#include "kernels.hpp"

#include <hip/hip_runtime.h>

namespace ellm {

// ---------------------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even; NaN stays NaN
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

// DPP lane permutations inside a row of 16 lanes
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
constexpr int DPP_QUAD_XOR1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int DPP_QUAD_XOR2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int DPP_ROW_HALF_MIRROR = 0x141; // lane i <-> 7 - i within each 8 lanes
constexpr int DPP_ROW_MIRROR = 0x140;      // lane i <-> 15 - i within each 16 lanes

// sum over the LPR (8 or 16) consecutive lanes that share one K row; every lane gets the sum
template <int LPR>
__device__ __forceinline__ float row_sum(float v) {
  v += dpp_f32<DPP_QUAD_XOR1>(v);
  v += dpp_f32<DPP_QUAD_XOR2>(v);
  v += dpp_f32<DPP_ROW_HALF_MIRROR>(v);
  if (LPR == 16) v += dpp_f32<DPP_ROW_MIRROR>(v);
  return v;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

constexpr float NEG_BIG = -1.0e30f;   // finite stand-in for "no score yet"; exp2(NEG_BIG - x) == 0

// ---------------------------------------------------------------------------------------------
// table patch: device_table[idx[i]] = val[i]
// ---------------------------------------------------------------------------------------------
__global__ void table_patch_kernel(int32_t* table, PatchArgs a) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < a.n) table[a.idx[i]] = a.val[i];
}

// ---------------------------------------------------------------------------------------------
// KV append: copy rows of D bf16 from the dense [token][Hkv][D] inputs to their chunk rows
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void kv_append_kernel(PoolView pv, const uint4* __restrict__ k_new,
                                                        const uint4* __restrict__ v_new, AppendArgs a) {
  constexpr int LPR = D * 2 / 16;            // lanes per row (16 bytes each)
  constexpr int ROWS = 256 / LPR;            // rows per block
  const int sub = threadIdx.x % LPR;
  const int64_t row = (int64_t)blockIdx.x * ROWS + threadIdx.x / LPR;
  const int64_t total_rows = (int64_t)a.total_new * pv.n_kv_heads * 2;
  if (row >= total_rows) return;
  const int per_tok = pv.n_kv_heads * 2;
  const int32_t tau = (int32_t)(row / per_tok);       // index of the new token in the launch
  const int rem = (int)(row - (int64_t)tau * per_tok);
  const int h = rem >> 1, plane = rem & 1;
  // request that owns token tau: largest b with tok0[b] <= tau
  int lo = 0, hi = a.n_req - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (a.tok0[mid] <= tau) lo = mid; else hi = mid - 1;
  }
  const int b = lo;
  const int64_t pos = (int64_t)a.len_before[b] + (tau - a.tok0[b]);
  const int32_t slot = (int32_t)(pos / pv.tokens_per_chunk);
  const int32_t r = (int32_t)(pos - (int64_t)slot * pv.tokens_per_chunk);
  const int32_t chunk = pv.table[(int64_t)a.tensor[b] * pv.max_slots + slot];
  const uint4* src = (plane ? v_new : k_new) + ((int64_t)tau * pv.n_kv_heads + h) * LPR + sub;
  char* dst = pv.base + (uint64_t)chunk * pv.chunk_bytes +
              ((uint64_t)(h * 2 + plane) * pv.tokens_per_chunk + r) * (D * 2) + sub * 16;
  *reinterpret_cast<uint4*>(dst) = *src;
}

// ---------------------------------------------------------------------------------------------
// decode attention, partial pass (split-K)
//
// One workgroup (4 waves) per (work item, kv head). A work item is a token range [t0, t1) of one
// request, at most split_tokens long. A K or V row of D bf16 is read by LPR = D/8 consecutive
// lanes with one 128-bit load each, so one wave-wide load covers RPW = 64/LPR consecutive rows
// (1 KiB, contiguous inside a chunk). Each lane keeps, for the G query heads of the group, the
// dot-product slice of its 8 dims; a DPP butterfly over the LPR lanes completes the score. The
// online softmax state (running max m, running sum l, weighted-V accumulator for the lane's 8
// dims) is per lane row-group; row-groups are merged with wave shuffles at the end, waves through
// LDS, and the merged (m, l, acc) goes to the workspace for the combine pass.
// Scores are kept in log2 units: q is pre-multiplied by scale * log2(e).
// ---------------------------------------------------------------------------------------------
template <int D, int G>
__global__ __launch_bounds__(256) void decode_partial_kernel(PoolView pv, const uint16_t* __restrict__ q,
                                                             float* __restrict__ ws, float scale_log2,
                                                             int32_t split_tokens, int32_t g_first,
                                                             BatchArgs a) {
  constexpr int LPR = D / 8;       // lanes per row
  constexpr int RPW = 64 / LPR;    // rows per wave-wide load
  constexpr int U = 4;             // loads in flight per lane and plane
  constexpr int TB = RPW * U;      // tokens per wave block
  constexpr int ROWB = D * 2;      // bytes per row

  __shared__ float sm_acc[4][G][D];
  __shared__ float sm_ml[4][G][2];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPR, rg = lane / LPR;
  const int item = blockIdx.x;
  const int g = blockIdx.y;                           // kv head
  const int hq0 = g * pv.group + g_first;            // first q head handled here

  // request of this item: number of item0[] entries <= item, minus one
  const int b = __syncthreads_count(tid < a.n_req && a.item0[tid] <= item) - 1;
  const int32_t tensor = a.tensor[b];
  const int32_t len = a.len[b];
  const int32_t t0 = (item - a.item0[b]) * split_tokens;
  const int32_t t1 = min(len, t0 + split_tokens);

  // q slice of this lane: 8 dims of each of the G heads, pre-scaled
  float qf[G][8];
  {
    const uint16_t* qb = q + ((int64_t)(a.q_row0 + b) * pv.n_q_heads + hq0) * D + sub * 8;
#pragma unroll
    for (int i = 0; i < G; i++) {
      uint4 w = *reinterpret_cast<const uint4*>(qb + i * D);
      qf[i][0] = bf16_lo(w.x) * scale_log2; qf[i][1] = bf16_hi(w.x) * scale_log2;
      qf[i][2] = bf16_lo(w.y) * scale_log2; qf[i][3] = bf16_hi(w.y) * scale_log2;
      qf[i][4] = bf16_lo(w.z) * scale_log2; qf[i][5] = bf16_hi(w.z) * scale_log2;
      qf[i][6] = bf16_lo(w.w) * scale_log2; qf[i][7] = bf16_hi(w.w) * scale_log2;
    }
  }

  float m[G], l[G], acc[G][8];
#pragma unroll
  for (int i = 0; i < G; i++) {
    m[i] = NEG_BIG; l[i] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; e++) acc[i][e] = 0.f;
  }

  // walk the chunks the token range touches; wave blocks are dealt round-robin over the 4 waves
  const int32_t Tc = pv.tokens_per_chunk;
  int32_t slot = t0 / Tc;
  int32_t r_begin = t0 - slot * Tc;
  int32_t remaining = t1 - t0;
  int32_t blk = 0;
  const int32_t* trow = pv.table + (int64_t)tensor * pv.max_slots;
  while (remaining > 0) {
    const int32_t rows = min(Tc - r_begin, remaining);
    const int32_t chunk = trow[slot];
    const char* kbase = pv.base + (uint64_t)chunk * pv.chunk_bytes +
                        ((uint64_t)(g * 2) * Tc + r_begin) * ROWB;
    const char* vbase = kbase + (uint64_t)Tc * ROWB;
    const int32_t nblk = (rows + TB - 1) / TB;
    for (int32_t ib = (wave - blk) & 3; ib < nblk; ib += 4) {
      uint4 kr[U], vr[U];
      bool ok[U];
#pragma unroll
      for (int u = 0; u < U; u++) {
        const int32_t rr = ib * TB + u * RPW + rg;
        ok[u] = rr < rows;
        const uint32_t off = (uint32_t)rr * ROWB + sub * 16;
        kr[u] = make_uint4(0, 0, 0, 0);
        vr[u] = make_uint4(0, 0, 0, 0);
        if (ok[u]) {
          kr[u] = *reinterpret_cast<const uint4*>(kbase + off);
          vr[u] = *reinterpret_cast<const uint4*>(vbase + off);
        }
      }
      float s[U][G];
#pragma unroll
      for (int u = 0; u < U; u++) {
        float kf[8] = {bf16_lo(kr[u].x), bf16_hi(kr[u].x), bf16_lo(kr[u].y), bf16_hi(kr[u].y),
                       bf16_lo(kr[u].z), bf16_hi(kr[u].z), bf16_lo(kr[u].w), bf16_hi(kr[u].w)};
#pragma unroll
        for (int i = 0; i < G; i++) {
          float d = 0.f;
#pragma unroll
          for (int e = 0; e < 8; e++) d = fmaf(qf[i][e], kf[e], d);
          d = row_sum<LPR>(d);
          s[u][i] = ok[u] ? d : -INFINITY;
        }
      }
#pragma unroll
      for (int i = 0; i < G; i++) {
        float mn = m[i];
#pragma unroll
        for (int u = 0; u < U; u++) mn = fmaxf(mn, s[u][i]);
        const float alpha = fast_exp2(m[i] - mn);
        m[i] = mn;
        l[i] *= alpha;
#pragma unroll
        for (int e = 0; e < 8; e++) acc[i][e] *= alpha;
#pragma unroll
        for (int u = 0; u < U; u++) s[u][i] = fast_exp2(s[u][i] - mn);
      }
#pragma unroll
      for (int u = 0; u < U; u++) {
        float vf[8] = {bf16_lo(vr[u].x), bf16_hi(vr[u].x), bf16_lo(vr[u].y), bf16_hi(vr[u].y),
                       bf16_lo(vr[u].z), bf16_hi(vr[u].z), bf16_lo(vr[u].w), bf16_hi(vr[u].w)};
#pragma unroll
        for (int i = 0; i < G; i++) {
          const float p = s[u][i];
          l[i] += p;
#pragma unroll
          for (int e = 0; e < 8; e++) acc[i][e] = fmaf(p, vf[e], acc[i][e]);
        }
      }
    }
    blk += nblk;
    remaining -= rows;
    slot += 1;
    r_begin = 0;
  }

  // merge the RPW row-groups of the wave (lanes that hold the same dims)
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
    for (int i = 0; i < G; i++) {
      const float mo = __shfl_xor(m[i], off);
      const float lo = __shfl_xor(l[i], off);
      const float mn = fmaxf(m[i], mo);
      const float ca = fast_exp2(m[i] - mn), cb = fast_exp2(mo - mn);
      l[i] = l[i] * ca + lo * cb;
#pragma unroll
      for (int e = 0; e < 8; e++) {
        const float ao = __shfl_xor(acc[i][e], off);
        acc[i][e] = acc[i][e] * ca + ao * cb;
      }
      m[i] = mn;
    }
  }
  if (rg == 0) {
#pragma unroll
    for (int i = 0; i < G; i++) {
      float4* dst = reinterpret_cast<float4*>(&sm_acc[wave][i][sub * 8]);
      dst[0] = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
      dst[1] = make_float4(acc[i][4], acc[i][5], acc[i][6], acc[i][7]);
      if (sub == 0) { sm_ml[wave][i][0] = m[i]; sm_ml[wave][i][1] = l[i]; }
    }
  }
  __syncthreads();
  // merge the 4 waves and write the partial: [item][q head][D + 2] = acc..., m, l
  float* wout = ws + ((int64_t)(a.item_base + item) * pv.n_q_heads + hq0) * (D + 2);
  for (int idx = tid; idx < G * D; idx += 256) {
    const int i = idx / D, d = idx - i * D;
    float mn = sm_ml[0][i][0];
#pragma unroll
    for (int w = 1; w < 4; w++) mn = fmaxf(mn, sm_ml[w][i][0]);
    float lsum = 0.f, asum = 0.f;
#pragma unroll
    for (int w = 0; w < 4; w++) {
      const float c = fast_exp2(sm_ml[w][i][0] - mn);
      lsum += sm_ml[w][i][1] * c;
      asum += sm_acc[w][i][d] * c;
    }
    wout[i * (D + 2) + d] = asum;
    if (d == 0) { wout[i * (D + 2) + D] = mn; wout[i * (D + 2) + D + 1] = lsum; }
  }
}

// ---------------------------------------------------------------------------------------------
// combine pass: merge the partials of every (request, q head) in split order, normalise, round
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(D) void decode_combine_kernel(const float* __restrict__ ws, uint16_t* __restrict__ out,
                                                           int32_t n_q_heads, BatchArgs a) {
  const int b = blockIdx.x, h = blockIdx.y, d = threadIdx.x;
  const int j0 = a.item0[b];
  const int j1 = (b + 1 < a.n_req) ? a.item0[b + 1] : a.n_items;
  float M = NEG_BIG, L = 0.f, A = 0.f;
  for (int j = j0; j < j1; j++) {
    const float* p = ws + ((int64_t)(a.item_base + j) * n_q_heads + h) * (D + 2);
    const float mj = p[D], lj = p[D + 1], aj = p[d];
    const float mn = fmaxf(M, mj);
    const float c0 = fast_exp2(M - mn), c1 = fast_exp2(mj - mn);
    L = L * c0 + lj * c1;
    A = A * c0 + aj * c1;
    M = mn;
  }
  out[((int64_t)(a.q_row0 + b) * n_q_heads + h) * D + d] = (uint16_t)f32_to_bf16_bits(A / L);
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
#define ELLM_HIP_CHECK_LAUNCH()                      \
  do {                                               \
    hipError_t e_ = hipGetLastError();               \
    if (e_ != hipSuccess) return (int)e_;            \
  } while (0)

int launch_table_patch(int32_t* table, const PatchArgs& a, hipStream_t stream) {
  if (a.n <= 0) return 0;
  hipLaunchKernelGGL(table_patch_kernel, dim3((a.n + 255) / 256), dim3(256), 0, stream, table, a);
  ELLM_HIP_CHECK_LAUNCH();
  return 0;
}

int launch_kv_append(const PoolView& pv, const void* k_new, const void* v_new, const AppendArgs& a,
                     hipStream_t stream) {
  if (a.total_new <= 0) return 0;
  const int64_t total_rows = (int64_t)a.total_new * pv.n_kv_heads * 2;
  if (pv.head_dim == 128) {
    const int64_t blocks = (total_rows + 15) / 16;
    hipLaunchKernelGGL(kv_append_kernel<128>, dim3((unsigned)blocks), dim3(256), 0, stream, pv,
                       (const uint4*)k_new, (const uint4*)v_new, a);
  } else {
    const int64_t blocks = (total_rows + 31) / 32;
    hipLaunchKernelGGL(kv_append_kernel<64>, dim3((unsigned)blocks), dim3(256), 0, stream, pv,
                       (const uint4*)k_new, (const uint4*)v_new, a);
  }
  ELLM_HIP_CHECK_LAUNCH();
  return 0;
}

template <int D, int G>
static void launch_partial_t(const PoolView& pv, const void* q, float* ws, float scale_log2, int32_t split_tokens,
                             int32_t g_first, const BatchArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL((decode_partial_kernel<D, G>), dim3(a.n_items, pv.n_kv_heads), dim3(256), 0, stream, pv,
                     (const uint16_t*)q, ws, scale_log2, split_tokens, g_first, a);
}

template <int D>
static int launch_partial_d(const PoolView& pv, const void* q, float* ws, float scale_log2, int32_t split_tokens,
                            const BatchArgs& a, hipStream_t stream) {
  // the q heads of a group are handled 8, 4, 2 or 1 at a time; a group size that is not one of
  // those is covered by several launches over the same K/V
  int done = 0;
  while (done < pv.group) {
    const int left = pv.group - done;
    if (left >= 8) { launch_partial_t<D, 8>(pv, q, ws, scale_log2, split_tokens, done, a, stream); done += 8; }
    else if (left >= 4) { launch_partial_t<D, 4>(pv, q, ws, scale_log2, split_tokens, done, a, stream); done += 4; }
    else if (left >= 2) { launch_partial_t<D, 2>(pv, q, ws, scale_log2, split_tokens, done, a, stream); done += 2; }
    else { launch_partial_t<D, 1>(pv, q, ws, scale_log2, split_tokens, done, a, stream); done += 1; }
    ELLM_HIP_CHECK_LAUNCH();
  }
  return 0;
}

int launch_decode(const PoolView& pv, const void* q, void* out, float* ws, float scale_log2, int32_t split_tokens,
                  const BatchArgs& a, hipStream_t stream) {
  if (a.n_req <= 0) return 0;
  int rc = pv.head_dim == 128 ? launch_partial_d<128>(pv, q, ws, scale_log2, split_tokens, a, stream)
                              : launch_partial_d<64>(pv, q, ws, scale_log2, split_tokens, a, stream);
  if (rc) return rc;
  if (pv.head_dim == 128)
    hipLaunchKernelGGL(decode_combine_kernel<128>, dim3(a.n_req, pv.n_q_heads), dim3(128), 0, stream, ws,
                       (uint16_t*)out, pv.n_q_heads, a);
  else
    hipLaunchKernelGGL(decode_combine_kernel<64>, dim3(a.n_req, pv.n_q_heads), dim3(64), 0, stream, ws,
                       (uint16_t*)out, pv.n_q_heads, a);
  ELLM_HIP_CHECK_LAUNCH();
  return 0;
}

}  // namespace ellm
