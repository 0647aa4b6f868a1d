// HIP kernels for gfx950 (CDNA4, 64-wide wavefronts): paged-attention decode with a split over the
// context and its reduction, the KV append, the block gather / scatter used by swaps, and the small
// map-maintenance kernels.
//
// What the attention kernels compute is the paged KV-cache attention of the paper's Section 2.3 for the
// per-layer access pattern of Section 3.2:
//   out[b][h] = sum_t softmax_t(scale * <q[b][h], K[b][g][t]>) V[b][g][t],   t < ctx_b,  g = h / (Hq/Hkv).
//
// Data layout of one block (one layer): [K|V][kv_head][token][head_dim]; one (block, head) K or V tile is
// block_tokens * head_dim contiguous elements.  The decode is bound by HBM bandwidth: every KV byte of the
// layer is read exactly once, with 16-byte loads per lane that cover a tile in contiguous 1 KiB pieces.

#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "pie_internal.h"

namespace pie {

// ---------------------------------------------------------------------------------------------------
// small kernels
// ---------------------------------------------------------------------------------------------------

__global__ void k_fill_i32(int32_t* __restrict__ p, int32_t n, int32_t v) {
  const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

__global__ void k_map_patch(int32_t* __restrict__ map, const MapPatch patch) {
  const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < patch.n) map[patch.handle[i]] = patch.slot[i];
}

int launch_map_fill(int32_t* d_map, int32_t n, int32_t value, hipStream_t s) {
  if (n <= 0) return PIE_OK;
  hipLaunchKernelGGL(k_fill_i32, dim3((n + 255) / 256), dim3(256), 0, s, d_map, n, value);
  PIE_HIP(hipGetLastError());
  return PIE_OK;
}

int launch_zero_u32(uint32_t* d, int32_t n, hipStream_t s) {
  return launch_map_fill(reinterpret_cast<int32_t*>(d), n, 0, s);
}

int launch_map_patch(int32_t* d_map, const MapPatch& patch, hipStream_t s) {
  if (patch.n <= 0) return PIE_OK;
  hipLaunchKernelGGL(k_map_patch, dim3((patch.n + 255) / 256), dim3(256), 0, s, d_map, patch);
  PIE_HIP(hipGetLastError());
  return PIE_OK;
}

// ---------------------------------------------------------------------------------------------------
// block gather / scatter (swap path PIE_SWAP_KERNEL)
//
// Copies pairs.n blocks of block_bytes each: dst_base + dst[i]*block_bytes <- src_base + src[i]*block_bytes.
// Either side may be pinned host memory mapped into the device's address space, so the kernel is bound by
// the host link: what matters is the number of 16-byte requests in flight, not the number of CUs.  A fixed,
// small grid strides over 4 KiB pieces; each lane keeps four loads in flight.
// ---------------------------------------------------------------------------------------------------

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kSwapThreads = 256;
constexpr int kSwapUnroll = 4;
constexpr size_t kSwapPiece = (size_t)kSwapThreads * 16 * kSwapUnroll;  // 16 KiB per workgroup iteration

__global__ __launch_bounds__(kSwapThreads) void k_swap_copy(char* __restrict__ dst_base,
                                                            const char* __restrict__ src_base, size_t block_bytes,
                                                            const SwapPairs pairs) {
  const size_t pieces_per_block = (block_bytes + kSwapPiece - 1) / kSwapPiece;
  const size_t n_pieces = pieces_per_block * (size_t)pairs.n;
  for (size_t piece = blockIdx.x; piece < n_pieces; piece += gridDim.x) {
    const int32_t i = (int32_t)(piece / pieces_per_block);
    const size_t off = (piece % pieces_per_block) * kSwapPiece;
    const u32x4* s = reinterpret_cast<const u32x4*>(src_base + (size_t)pairs.src[i] * block_bytes + off);
    u32x4* d = reinterpret_cast<u32x4*>(dst_base + (size_t)pairs.dst[i] * block_bytes + off);
    const size_t n16 = (block_bytes - off < kSwapPiece ? block_bytes - off : kSwapPiece) / 16;
    u32x4 v[kSwapUnroll];
#pragma unroll
    for (int u = 0; u < kSwapUnroll; ++u) {
      const size_t j = (size_t)u * kSwapThreads + threadIdx.x;
      if (j < n16) v[u] = __builtin_nontemporal_load(s + j);
    }
#pragma unroll
    for (int u = 0; u < kSwapUnroll; ++u) {
      const size_t j = (size_t)u * kSwapThreads + threadIdx.x;
      if (j < n16) __builtin_nontemporal_store(v[u], d + j);
    }
  }
}

int launch_swap_copy(char* dst_layer_base, const char* src_layer_base, size_t block_bytes, const SwapPairs& pairs,
                     int n_wgs, hipStream_t s) {
  if (pairs.n <= 0) return PIE_OK;
  if (block_bytes % 16) return PIE_EINVAL;
  const size_t pieces = ((block_bytes + kSwapPiece - 1) / kSwapPiece) * (size_t)pairs.n;
  const int grid = (int)(pieces < (size_t)n_wgs ? pieces : (size_t)n_wgs);
  hipLaunchKernelGGL(k_swap_copy, dim3(grid), dim3(kSwapThreads), 0, s, dst_layer_base, src_layer_base, block_bytes,
                     pairs);
  PIE_HIP(hipGetLastError());
  return PIE_OK;
}

// ---------------------------------------------------------------------------------------------------
// element types
// ---------------------------------------------------------------------------------------------------

struct F32 { using T = float; };
struct F16 { using T = uint16_t; };
struct BF16 { using T = uint16_t; };

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);                                            // nearest even
  return (uint16_t)(u >> 16);
}

template <typename E> struct Elem;
template <> struct Elem<F32> {
  static constexpr int kVec = 4;  // elements in 16 bytes
  __device__ static void unpack(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y); f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
  __device__ static void store(void* base, size_t idx, float v) { reinterpret_cast<float*>(base)[idx] = v; }
};
template <> struct Elem<F16> {
  static constexpr int kVec = 8;
  __device__ static void unpack(const uint4& r, float* f) {
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __half2float(__ushort_as_half((unsigned short)(w[i] & 0xffffu)));
      f[2 * i + 1] = __half2float(__ushort_as_half((unsigned short)(w[i] >> 16)));
    }
  }
  __device__ static void store(void* base, size_t idx, float v) {
    reinterpret_cast<__half*>(base)[idx] = __float2half_rn(v);
  }
};
template <> struct Elem<BF16> {
  static constexpr int kVec = 8;
  __device__ static void unpack(const uint4& r, float* f) {
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  __device__ static void store(void* base, size_t idx, float v) {
    reinterpret_cast<uint16_t*>(base)[idx] = f32_to_bf16_bits(v);
  }
};

// ---------------------------------------------------------------------------------------------------
// handle -> device slot, with the checks that keep a bad table from becoming a bad address
// ---------------------------------------------------------------------------------------------------

__device__ __forceinline__ int32_t resolve_slot(int32_t handle, const int32_t* __restrict__ map, int32_t n_handles,
                                                int32_t n_gpu_blocks, int32_t n_slots, bool stage_valid,
                                                uint32_t* __restrict__ err) {
  if (handle < 0 || handle >= n_handles) {
    atomicOr(err, PIE_DEVERR_BAD_HANDLE);
    return -1;
  }
  const int32_t slot = map[handle];
  if (slot < 0 || slot >= n_slots || (slot >= n_gpu_blocks && !stage_valid)) {
    atomicOr(err, PIE_DEVERR_NOT_PRESENT);
    return -1;
  }
  return slot;
}

// ---------------------------------------------------------------------------------------------------
// KV append: one workgroup per sequence copies the new token's key and value rows into its tail block
// ---------------------------------------------------------------------------------------------------

struct AppendArgs {
  char* kv_layer;            // device pool base of this layer
  const int32_t* map;
  uint32_t* err;
  const char* k_new;         // [B][Hkv][d]
  const char* v_new;
  const int32_t* table;
  const int32_t* ctx;
  size_t block_bytes;
  int32_t max_blocks, n_handles, n_gpu_blocks, n_slots, n_kv_heads, head_dim, block_tokens, elem_bytes;
  int32_t stage_valid;
};

__global__ __launch_bounds__(256) void k_kv_append(const AppendArgs a) {
  const int32_t b = blockIdx.x;
  const int32_t ctx = a.ctx[b];
  if (ctx <= 0) return;
  const int32_t pos = ctx - 1;
  const int32_t j = pos / a.block_tokens;
  if (j >= a.max_blocks) {
    if (threadIdx.x == 0) atomicOr(a.err, PIE_DEVERR_BAD_HANDLE);
    return;
  }
  __shared__ int32_t s_slot;
  if (threadIdx.x == 0)
    s_slot = resolve_slot(a.table[(size_t)b * a.max_blocks + j], a.map, a.n_handles, a.n_gpu_blocks, a.n_slots,
                          a.stage_valid != 0, a.err);
  __syncthreads();
  const int32_t slot = s_slot;
  if (slot < 0) return;
  const int32_t row_bytes = a.head_dim * a.elem_bytes;              // multiple of 16
  const int32_t vec_per_row = row_bytes / 16;
  const int32_t n_vec = a.n_kv_heads * vec_per_row;
  char* blk = a.kv_layer + (size_t)slot * a.block_bytes;
  const size_t v_off = a.block_bytes / 2;
  const int32_t t = pos % a.block_tokens;
  for (int32_t i = threadIdx.x; i < n_vec; i += blockDim.x) {
    const int32_t g = i / vec_per_row, c = i % vec_per_row;
    const size_t src = ((size_t)b * a.n_kv_heads + g) * row_bytes + (size_t)c * 16;
    const size_t dst = ((size_t)g * a.block_tokens + t) * row_bytes + (size_t)c * 16;
    *reinterpret_cast<uint4*>(blk + dst) = *reinterpret_cast<const uint4*>(a.k_new + src);
    *reinterpret_cast<uint4*>(blk + v_off + dst) = *reinterpret_cast<const uint4*>(a.v_new + src);
  }
}

int launch_kv_append(const pie_pool* p, int32_t layer, const void* d_k, const void* d_v, const int32_t* d_table,
                     int32_t max_blocks, const int32_t* d_ctx, int32_t batch, bool stage_valid, hipStream_t s) {
  if (((uintptr_t)d_k | (uintptr_t)d_v) % 16) return PIE_EINVAL;
  AppendArgs a;
  a.kv_layer = p->d_kv + (size_t)layer * p->d_layer_stride;
  a.map = p->d_map[layer & 1];
  a.err = p->d_err;
  a.k_new = (const char*)d_k;
  a.v_new = (const char*)d_v;
  a.table = d_table;
  a.ctx = d_ctx;
  a.block_bytes = p->block_bytes;
  a.max_blocks = max_blocks;
  a.n_handles = p->n_handles;
  a.n_gpu_blocks = p->cfg.n_gpu_blocks;
  a.n_slots = p->cfg.n_gpu_blocks + 2 * p->cfg.n_stage_blocks;
  a.n_kv_heads = p->cfg.n_kv_heads;
  a.head_dim = p->cfg.head_dim;
  a.block_tokens = p->cfg.block_tokens;
  a.elem_bytes = p->elem_bytes;
  a.stage_valid = stage_valid ? 1 : 0;
  hipLaunchKernelGGL(k_kv_append, dim3(batch), dim3(256), 0, s, a);
  PIE_HIP(hipGetLastError());
  return PIE_OK;
}

// ---------------------------------------------------------------------------------------------------
// paged-attention decode
//
// Grid (partition, kv_head, sequence); a workgroup of kWaves wavefronts handles `part_tokens` tokens of
// one (sequence, kv head) and all G query heads that share it.  Wave w takes blocks w, w + kWaves, ... of
// the partition.  A tile (16 tokens x head_dim) is read with NLD loads of 16 bytes per lane: LPR lanes
// cover one token row, so a wave-wide load covers TPL = 64 / LPR consecutive tokens = 1 KiB contiguous.
// Lane (rg, c) = (lane / LPR, lane % LPR) owns head dims [c*VEC, (c+1)*VEC) of tokens rg, rg + TPL, ...
//
// Each of the TPL row groups runs its own online softmax (running max m, sum l, accumulator acc) over the
// tokens it owns, in the log2 domain (scores are pre-multiplied by scale*log2(e)).  The only cross-lane
// traffic in the loop is the sum of the partial dot products over the LPR lanes of a row.  At the end the
// kWaves*TPL partial states are merged through LDS, then either written out (single partition) or stored
// as (m, l, acc) for the reduction kernel.
// ---------------------------------------------------------------------------------------------------

#ifndef PIE_KWAVES
#define PIE_KWAVES 4
#endif
constexpr int kWaves = PIE_KWAVES;
constexpr int kBlockTokens = 16;
constexpr float kNegBig = -1.0e30f;   // finite stand-in for -inf as the initial running max

template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false);
  return x + __int_as_float(y);
}

// Sum over the LPR consecutive lanes of a row; every lane of the row gets the total.
template <int LPR>
__device__ __forceinline__ float row_sum(float x) {
  x = dpp_add<0xB1>(x);                      // quad_perm [1,0,3,2]: lane ^ 1
  x = dpp_add<0x4E>(x);                      // quad_perm [2,3,0,1]: lane ^ 2
  if (LPR >= 8) x = dpp_add<0x141>(x);       // row_half_mirror: the other quad of the 8
  if (LPR >= 16) x = dpp_add<0x140>(x);      // row_mirror: the other half of the 16
  if (LPR >= 32) x += __shfl_xor(x, 16, 64);
  if (LPR >= 64) x += __shfl_xor(x, 32, 64);
  return x;
}

struct AttnArgs {
  const char* kv_layer;
  const int32_t* map;
  uint32_t* err;
  const char* q;             // [B][Hq][d]
  char* out;                 // [B][Hq][d]
  float* ws;                 // [B][Hq][n_parts][2 + d]
  const int32_t* table;
  const int32_t* ctx;
  size_t block_bytes;
  float scale_log2e;
  int32_t max_blocks, n_handles, n_gpu_blocks, n_slots, n_kv_heads, part_tokens, n_parts;
  int32_t stage_valid;
  int32_t nontemporal;       // stream K/V past the caches (each byte is read once)
  int32_t exp_mode;          // TIMING EXPERIMENT ONLY
#ifdef PIE_EXPERIMENT
  unsigned long long* dbg;   // per-workgroup timestamps
  int32_t dbg_cap;
#endif
};

__device__ __forceinline__ uint4 nt_load16(const char* p) {
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

template <typename E, int HD, int G, bool NT>
__global__ __launch_bounds__(kWaves * 64) void k_attn_decode(const AttnArgs a) {
  using EL = Elem<E>;
  constexpr int VEC = EL::kVec;
  constexpr int LPR = HD / VEC;
  constexpr int TPL = 64 / LPR;
  constexpr int NLD = kBlockTokens / TPL;
  constexpr int TILE_BYTES = kBlockTokens * HD * (16 / VEC);
  static_assert(LPR >= 4 && LPR <= 64 && NLD >= 1, "unsupported head_dim / dtype");

  // grid (kv head, sequence, partition): partitions are the slowest index, so the short last partitions of
  // the sequences are dispatched at the end and even out the tail of the launch
  const int32_t g = blockIdx.x, b = blockIdx.y, part = blockIdx.z;
#ifdef PIE_EXPERIMENT
  const unsigned long long t_entry = wall_clock64();
#endif
  const int32_t ctx = a.ctx[b];
  const int32_t tok0 = part * a.part_tokens;
  const int32_t n_parts_b = ctx <= 0 ? 1 : (ctx + a.part_tokens - 1) / a.part_tokens;
  if (part >= n_parts_b) return;
  const int32_t tok1 = min(ctx, tok0 + a.part_tokens);           // may be <= tok0 only when ctx <= 0
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int rg = lane / LPR, c = lane % LPR;
  const int32_t hq0 = g * G;
  const int32_t n_q_heads = a.n_kv_heads * G;

  // query rows of the G heads, this lane's VEC dims, as fp32 pre-multiplied by scale*log2(e)
  float q[G][VEC];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    const uint4 r = *reinterpret_cast<const uint4*>(a.q + (((size_t)b * n_q_heads + hq0 + h) * HD + c * VEC) * (16 / VEC));
    EL::unpack(r, q[h]);
#pragma unroll
    for (int v = 0; v < VEC; ++v) q[h][v] *= a.scale_log2e;
  }

  float m[G], l[G], acc[G][VEC];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    m[h] = kNegBig;
    l[h] = 0.f;
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[h][v] = 0.f;
  }

  // blocks of this partition handled by this wave: j = jb0 + wave + kWaves * it
  const int32_t jb0 = tok0 / kBlockTokens;
  const int32_t jb1 = (tok1 + kBlockTokens - 1) / kBlockTokens;   // exclusive
  const int32_t n_it = (jb1 - jb0 - wave + kWaves - 1) / kWaves;  // <= part_tokens / (16 * kWaves) <= 64

  // each lane resolves the slot of one of the wave's blocks up front (dependent loads off the hot loop)
  int32_t my_slot = -1;
  if (lane < n_it) {
    const int32_t j = jb0 + wave + kWaves * lane;
    my_slot = j < a.max_blocks ? resolve_slot(a.table[(size_t)b * a.max_blocks + j], a.map, a.n_handles,
                                              a.n_gpu_blocks, a.n_slots, a.stage_valid != 0, a.err)
                               : -1;
    if (j >= a.max_blocks) atomicOr(a.err, PIE_DEVERR_BAD_HANDLE);
  }

  // TIMING EXPERIMENT (exp_mode & 4): pretend K and V tiles of a head are adjacent (in-bounds, wrong data)
  const size_t head_off = (a.exp_mode & 4) ? (size_t)g * 2 * TILE_BYTES : (size_t)g * TILE_BYTES;
  const size_t v_off = (a.exp_mode & 4) ? (size_t)TILE_BYTES : a.block_bytes / 2;

  // Two register sets: while one tile is consumed the next is already in flight (8 KiB per wave).
  uint4 kA[NLD], vA[NLD], kB[NLD], vB[NLD];
  auto load_tile = [&](uint4 (&kr)[NLD], uint4 (&vr)[NLD], int32_t it) {
    int32_t slot = __shfl(my_slot, it, 64);
    slot = slot < 0 ? 0 : slot;                                    // flagged blocks are masked below
    const char* kp = a.kv_layer + (size_t)slot * a.block_bytes + head_off + (size_t)lane * 16;
#pragma unroll
    for (int i = 0; i < NLD; ++i) kr[i] = NT ? nt_load16(kp + (size_t)i * 1024)
                                             : *reinterpret_cast<const uint4*>(kp + (size_t)i * 1024);
#pragma unroll
    for (int i = 0; i < NLD; ++i) vr[i] = NT ? nt_load16(kp + v_off + (size_t)i * 1024)
                                             : *reinterpret_cast<const uint4*>(kp + v_off + (size_t)i * 1024);
  };
  auto consume = [&](uint4 (&kr)[NLD], uint4 (&vr)[NLD], int32_t it) {
    const int32_t t_base = (jb0 + wave + kWaves * it) * kBlockTokens + rg;   // token of load 0
    const bool present = __shfl(my_slot, it, 64) >= 0;
    const int32_t limit = present ? tok1 : 0;                               // a missing block contributes nothing
    const bool tail = t_base - rg + kBlockTokens > limit;

    float s[G][NLD];
    if (a.exp_mode & 1) {
      uint32_t x = 0;
#pragma unroll
      for (int i = 0; i < NLD; ++i) x ^= kr[i].x ^ kr[i].y ^ kr[i].z ^ kr[i].w;
#pragma unroll
      for (int i = 0; i < NLD; ++i)
#pragma unroll
        for (int h = 0; h < G; ++h) s[h][i] = (x == 0x12345u) ? 1.f : 0.f;
    } else
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      float kf[VEC];
      EL::unpack(kr[i], kf);
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float d = 0.f;
#pragma unroll
        for (int v = 0; v < VEC; ++v) d = fmaf(q[h][v], kf[v], d);
        s[h][i] = row_sum<LPR>(d);
      }
    }
    if (tail) {
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const bool valid = t_base + i * TPL < limit;
#pragma unroll
        for (int h = 0; h < G; ++h) s[h][i] = valid ? s[h][i] : -INFINITY;
        if (!valid) vr[i] = make_uint4(0, 0, 0, 0);                // garbage rows must not reach the sum
      }
    }
    float p[G][NLD];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float mx = s[h][0];
#pragma unroll
      for (int i = 1; i < NLD; ++i) mx = fmaxf(mx, s[h][i]);
      const float m_new = fmaxf(m[h], mx);
      const float corr = __builtin_amdgcn_exp2f(m[h] - m_new);
      float ps = 0.f;
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        p[h][i] = __builtin_amdgcn_exp2f(s[h][i] - m_new);
        ps += p[h][i];
      }
      l[h] = l[h] * corr + ps;
      m[h] = m_new;
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[h][v] *= corr;
    }
    if (a.exp_mode & 2) {
      uint32_t x = 0;
#pragma unroll
      for (int i = 0; i < NLD; ++i) x ^= vr[i].x ^ vr[i].y ^ vr[i].z ^ vr[i].w;
      acc[0][0] += (x == 0x12345u) ? p[0][0] : 0.f;
    } else
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      float vf[VEC];
      EL::unpack(vr[i], vf);
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[h][v] = fmaf(p[h][i], vf[v], acc[h][v]);
    }
  };

#ifdef PIE_EXPERIMENT
  const unsigned long long t_pro = wall_clock64();
#endif
  if (n_it > 0) load_tile(kA, vA, 0);
  for (int32_t it = 0; it < n_it; it += 2) {
    if (it + 1 < n_it) load_tile(kB, vB, it + 1);
    consume(kA, vA, it);
    if (it + 1 < n_it) {
      if (it + 2 < n_it) load_tile(kA, vA, it + 2);
      consume(kB, vB, it + 1);
    }
  }

#ifdef PIE_EXPERIMENT
  const unsigned long long t_loop = wall_clock64();
#endif
  // merge the kWaves * TPL partial states, one query head at a time to keep LDS small
  constexpr int NP = kWaves * TPL;
  __shared__ float s_m[NP], s_l[NP];
  __shared__ float s_acc[NP][HD];
  const int pidx = wave * TPL + rg;
#pragma unroll
  for (int h = 0; h < G; ++h) {
    if (h > 0) __syncthreads();
    if (c == 0) {
      s_m[pidx] = m[h];
      s_l[pidx] = l[h];
    }
#pragma unroll
    for (int v = 0; v < VEC; ++v) s_acc[pidx][c * VEC + v] = acc[h][v];
    __syncthreads();
    for (int dim = threadIdx.x; dim < HD; dim += kWaves * 64) {
      float M = s_m[0];
#pragma unroll
      for (int i = 1; i < NP; ++i) M = fmaxf(M, s_m[i]);
      float L = 0.f, A = 0.f;
#pragma unroll
      for (int i = 0; i < NP; ++i) {
        const float w = __builtin_amdgcn_exp2f(s_m[i] - M);
        L = fmaf(w, s_l[i], L);
        A = fmaf(w, s_acc[i][dim], A);
      }
      const size_t row = (size_t)b * n_q_heads + hq0 + h;
      if (a.n_parts == 1) {
        EL::store(a.out, row * HD + dim, L > 0.f ? A / L : 0.f);
      } else {
        float* w = a.ws + (row * a.n_parts + part) * (HD + 2);
        if (dim == 0) {
          w[0] = M;
          w[1] = L;
        }
        w[2 + dim] = A;
      }
    }
  }
#ifdef PIE_EXPERIMENT
  if (a.dbg && lane == 0) {
    const int wg = (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
    if (wg < a.dbg_cap) {
      unsigned long long* d = a.dbg + ((size_t)wg * kWaves + wave) * 6;
      d[0] = t_entry; d[1] = t_pro; d[2] = t_loop; d[3] = wall_clock64();
      d[4] = (unsigned long long)n_it;
      unsigned hwid; asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hwid));
      unsigned xcc; asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
      d[5] = ((unsigned long long)xcc << 32) | hwid;
    }
  }
#endif
}

// Reduction over the partitions of one (sequence, query head): out = sum_s 2^(m_s - M) acc_s / sum_s 2^(m_s - M) l_s.
template <typename E, int HD>
__global__ __launch_bounds__(HD) void k_attn_reduce(const AttnArgs a, int32_t n_q_heads) {
  using EL = Elem<E>;
  const int32_t hq = blockIdx.x, b = blockIdx.y, dim = threadIdx.x;
  const int32_t ctx = a.ctx[b];
  int32_t np = ctx <= 0 ? 1 : (ctx + a.part_tokens - 1) / a.part_tokens;
  if (np > a.n_parts) np = a.n_parts;               // a context beyond the table's width was flagged upstream
  const size_t row = (size_t)b * n_q_heads + hq;
  const float* w = a.ws + row * a.n_parts * (HD + 2);
  float M = kNegBig;
  for (int32_t s = 0; s < np; ++s) M = fmaxf(M, w[(size_t)s * (HD + 2)]);
  float L = 0.f, A = 0.f;
  for (int32_t s = 0; s < np; ++s) {
    const float* ws = w + (size_t)s * (HD + 2);
    const float wt = __builtin_amdgcn_exp2f(ws[0] - M);
    L = fmaf(wt, ws[1], L);
    A = fmaf(wt, ws[2 + dim], A);
  }
  EL::store(a.out, row * HD + dim, L > 0.f ? A / L : 0.f);
}

// ---- dispatch ----------------------------------------------------------------------------------------

constexpr int kMinPartTokens = 256;

static bool pick(int32_t dtype, int32_t hd, int32_t g) {
  if (dtype < 0 || dtype > 2) return false;
  if (hd != 64 && hd != 128) return false;
  return g == 1 || g == 2 || g == 4 || g == 8;
}

bool attn_config_supported(const pie_config& c) {
  return c.block_tokens == kBlockTokens && pick(c.dtype, c.head_dim, c.n_q_heads / c.n_kv_heads);
}

size_t attn_workspace_floats(const pie_config& c) {
  const size_t max_parts = ((size_t)c.max_blocks_per_seq * c.block_tokens + kMinPartTokens - 1) / kMinPartTokens;
  return (size_t)c.max_batch * c.n_q_heads * (max_parts ? max_parts : 1) * (c.head_dim + 2);
}

template <typename E, int HD, int G>
static int launch_typed(const AttnArgs& a, int32_t batch, int32_t n_q_heads, hipStream_t s, hipEvent_t e0,
                        hipEvent_t e1) {
  if (e0) PIE_HIP(hipEventRecord(e0, s));
  if (a.nontemporal)
    hipLaunchKernelGGL((k_attn_decode<E, HD, G, true>), dim3(a.n_kv_heads, batch, a.n_parts), dim3(kWaves * 64), 0, s, a);
  else
    hipLaunchKernelGGL((k_attn_decode<E, HD, G, false>), dim3(a.n_kv_heads, batch, a.n_parts), dim3(kWaves * 64), 0, s, a);
  PIE_HIP(hipGetLastError());
  if (e1) PIE_HIP(hipEventRecord(e1, s));
  if (a.n_parts > 1) {
    hipLaunchKernelGGL((k_attn_reduce<E, HD>), dim3(n_q_heads, batch), dim3(HD), 0, s, a, n_q_heads);
    PIE_HIP(hipGetLastError());
  }
  return PIE_OK;
}

template <typename E, int HD>
static int launch_g(const AttnArgs& a, int32_t g, int32_t batch, int32_t nq, hipStream_t s, hipEvent_t e0,
                    hipEvent_t e1) {
  switch (g) {
    case 1: return launch_typed<E, HD, 1>(a, batch, nq, s, e0, e1);
    case 2: return launch_typed<E, HD, 2>(a, batch, nq, s, e0, e1);
    case 4: return launch_typed<E, HD, 4>(a, batch, nq, s, e0, e1);
    case 8: return launch_typed<E, HD, 8>(a, batch, nq, s, e0, e1);
    default: return PIE_EINVAL;
  }
}

template <typename E>
static int launch_hd(const AttnArgs& a, int32_t hd, int32_t g, int32_t batch, int32_t nq, hipStream_t s, hipEvent_t e0,
                     hipEvent_t e1) {
  switch (hd) {
    case 64: return launch_g<E, 64>(a, g, batch, nq, s, e0, e1);
    case 128: return launch_g<E, 128>(a, g, batch, nq, s, e0, e1);
    default: return PIE_EINVAL;
  }
}

int launch_attn_decode(const pie_pool* p, int32_t layer, const void* d_q, const int32_t* d_table, int32_t max_blocks,
                       const int32_t* d_ctx, int32_t batch, void* d_out, bool stage_valid, hipStream_t s,
                       hipEvent_t k_start, hipEvent_t k_end) {
  const pie_config& c = p->cfg;
  if (((uintptr_t)d_q | (uintptr_t)d_out) % 16) return PIE_EINVAL;
  if (max_blocks <= 0) return PIE_EINVAL;
  const int32_t g = c.n_q_heads / c.n_kv_heads;
  // partition size: a multiple of one pass of the workgroup's waves, at most 64 blocks per wave
  int32_t part = p->attn_partition;
  const int32_t quantum = kWaves * kBlockTokens;
  if (part < kMinPartTokens) part = kMinPartTokens;
  part = (part + quantum - 1) / quantum * quantum;
  if (part > quantum * 64) part = quantum * 64;
  const int32_t max_tokens = max_blocks * kBlockTokens;
  int32_t n_parts = (max_tokens + part - 1) / part;
  if ((size_t)batch * c.n_q_heads * n_parts * (c.head_dim + 2) > p->ws_floats) return PIE_ENOMEM;

  AttnArgs a;
  a.kv_layer = p->d_kv + (size_t)layer * p->d_layer_stride;
  a.map = p->d_map[layer & 1];
  a.err = p->d_err;
  a.q = (const char*)d_q;
  a.out = (char*)d_out;
  a.ws = p->d_ws;
  a.table = d_table;
  a.ctx = d_ctx;
  a.block_bytes = p->block_bytes;
  a.scale_log2e = p->scale_log2e;
  a.max_blocks = max_blocks;
  a.n_handles = p->n_handles;
  a.n_gpu_blocks = c.n_gpu_blocks;
  a.n_slots = c.n_gpu_blocks + 2 * c.n_stage_blocks;
  a.n_kv_heads = c.n_kv_heads;
  a.part_tokens = part;
  a.n_parts = n_parts;
  a.stage_valid = stage_valid ? 1 : 0;
  a.nontemporal = p->attn_nontemporal ? 1 : 0;
  { const char* e = getenv("PIE_EXP_MODE"); a.exp_mode = e ? atoi(e) : 0; }
#ifdef PIE_EXPERIMENT
  { const char* e = getenv("PIE_DBG_PTR"); a.dbg = e ? (unsigned long long*)strtoull(e, nullptr, 10) : nullptr;
    const char* c2 = getenv("PIE_DBG_CAP"); a.dbg_cap = c2 ? atoi(c2) : 0; }
#endif
  if (a.n_slots <= 0) return PIE_EINVAL;
  switch (c.dtype) {
    case PIE_DTYPE_F32: return launch_hd<F32>(a, c.head_dim, g, batch, c.n_q_heads, s, k_start, k_end);
    case PIE_DTYPE_F16: return launch_hd<F16>(a, c.head_dim, g, batch, c.n_q_heads, s, k_start, k_end);
    case PIE_DTYPE_BF16: return launch_hd<BF16>(a, c.head_dim, g, batch, c.n_q_heads, s, k_start, k_end);
    default: return PIE_EINVAL;
  }
}

}  // namespace pie
