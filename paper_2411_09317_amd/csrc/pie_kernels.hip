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
// Work is cut into items: `part_tokens` consecutive tokens of one sequence.  A small planning kernel lists
// the non-empty items, full ones first and the sequences' shorter last pieces after them in descending
// size, and a resolve kernel turns the block table (handles) into device slots once per step.  The decode
// kernel is persistent: about as many workgroups as the GPU can hold resident, each taking (item, kv head)
// units from an atomic ticket counter until none are left.  That evens out the 8 XCDs (which do not stream
// at the same rate), leaves only small units for the end of the launch, and pays the launch ramp once.
//
// A workgroup of kWaves wavefronts handles one unit and all G query heads that share the kv head.  Wave w
// takes blocks w, w + kWaves, ... of the item.  A tile (16 tokens x head_dim) is read with NLD loads of 16
// bytes per lane: LPR lanes cover one token row, so a wave-wide load covers TPL = 64 / LPR consecutive tokens
// = 1 KiB contiguous.  Lane (rg, c) = (lane / LPR, lane % LPR) owns head dims [c*VEC, (c+1)*VEC) of tokens
// rg, rg + TPL, ...  Loads are non-temporal (every KV byte is read once) and double-buffered in registers.
//
// Each of the TPL row groups runs its own online softmax (running max m, sum l, accumulator acc) over the
// tokens it owns, in the log2 domain (scores are pre-multiplied by scale*log2(e)).  The only cross-lane
// traffic in the loop is the sum of the partial dot products over the LPR lanes of a row.  At the end the
// kWaves*TPL partial states are merged through LDS, then either written out (single partition) or stored
// as (m, l, acc) for the reduction kernel.
// ---------------------------------------------------------------------------------------------------

constexpr int kWaves = 4;
constexpr int kBlockTokens = 16;
constexpr int kMinPartTokens = 256;
constexpr int kMaxPlanBatch = 4096;   // sequences the planning kernel keeps in LDS
constexpr int kPlanHdrInts = 16;
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

__device__ __forceinline__ uint4 nt_load16(const char* p) {
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// Context length as the kernels use it: never beyond what the block table can name.
__device__ __forceinline__ int32_t clamp_ctx(int32_t ctx, int32_t max_blocks) {
  const int32_t cap = max_blocks * kBlockTokens;
  return ctx > cap ? cap : ctx;
}

// ---- planning: the list of work items ------------------------------------------------------------------
// items[i] = {sequence | part << 16, end token of the item}.  hdr[0] = number of items.  Full items
// (part_tokens tokens) come first, then one shorter item per sequence whose length is not a multiple of
// part_tokens (or is <= 0, so that its output is still written), longest first.  Also zeroes the ticket
// counters of all layers.
__global__ __launch_bounds__(256) void k_attn_plan(const int32_t* __restrict__ ctx, int32_t batch, int32_t part_tokens,
                                                   int32_t max_blocks, uint2* __restrict__ items,
                                                   int32_t* __restrict__ hdr, uint32_t* __restrict__ counters,
                                                   int32_t n_counters, uint32_t* __restrict__ err) {
  __shared__ int32_t s_off[kMaxPlanBatch];   // first full item of the sequence
  __shared__ int32_t s_nf[kMaxPlanBatch];
  __shared__ int32_t s_rem[kMaxPlanBatch];   // size of the short item, -1 if none
  __shared__ int32_t s_total_full;
  for (int32_t b = threadIdx.x; b < batch; b += blockDim.x) {
    const int32_t raw = ctx[b];
    const int32_t c = clamp_ctx(raw, max_blocks);
    if (raw > c) atomicOr(err, PIE_DEVERR_BAD_HANDLE);   // the table cannot name that many blocks
    const int32_t nf = c > 0 ? c / part_tokens : 0;
    const int32_t rem = c > 0 ? c % part_tokens : 0;
    s_nf[b] = nf;
    s_rem[b] = (rem > 0 || c <= 0) ? rem : -1;
  }
  for (int32_t i = threadIdx.x; i < n_counters; i += blockDim.x) counters[i] = 0;
  __syncthreads();
  if (threadIdx.x == 0) {
    int32_t off = 0, n_short = 0;
    for (int32_t b = 0; b < batch; ++b) {
      s_off[b] = off;
      off += s_nf[b];
      if (s_rem[b] >= 0) ++n_short;
    }
    s_total_full = off;
    hdr[0] = off + n_short;
  }
  __syncthreads();
  const int32_t total_full = s_total_full;
  for (int32_t b = threadIdx.x; b < batch; b += blockDim.x) {
    const int32_t nf = s_nf[b];
    for (int32_t p = 0; p < nf; ++p)
      items[s_off[b] + p] = make_uint2((uint32_t)b | ((uint32_t)p << 16), (uint32_t)((p + 1) * part_tokens));
    const int32_t key = s_rem[b];
    if (key >= 0) {
      int32_t rank = 0;                                  // longest first, ties by sequence index
      for (int32_t o = 0; o < batch; ++o) {
        const int32_t k2 = s_rem[o];
        rank += (k2 > key || (k2 == key && o < b)) ? 1 : 0;
      }
      items[total_full + rank] = make_uint2((uint32_t)b | ((uint32_t)nf << 16), (uint32_t)(nf * part_tokens + key));
    }
  }
}

// ---- resolve: the device slots of every item's blocks, for one or both staging regions ---------------------
// slots[r][i * bpi + jj] = slot of block (part * bpi + jj) of item i's sequence, -1 beyond its context.
struct ResolveArgs {
  const int32_t* table;      // [B][max_blocks] handles
  const uint2* items;
  const int32_t* hdr;
  const int32_t* map[2];
  int32_t* slots[2];         // NULL to skip a region
  uint32_t* err;
  int32_t max_blocks, n_handles, n_gpu_blocks, n_slots, blocks_per_item;
  int32_t stage_valid[2];
};

__global__ __launch_bounds__(64) void k_attn_resolve(const ResolveArgs a) {
  const int32_t i = blockIdx.x;
  if (i >= a.hdr[0]) return;
  const uint2 rec = a.items[i];
  const int32_t b = (int32_t)(rec.x & 0xffffu), part = (int32_t)(rec.x >> 16);
  const int32_t tok1 = (int32_t)rec.y;
  const int32_t jb1 = tok1 > 0 ? (tok1 + kBlockTokens - 1) / kBlockTokens : 0;   // <= max_blocks
  for (int32_t jj = threadIdx.x; jj < a.blocks_per_item; jj += blockDim.x) {
    const int32_t j = part * a.blocks_per_item + jj;
    const bool live = j < jb1;
    const int32_t h = live ? a.table[(size_t)b * a.max_blocks + j] : -1;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      if (!a.slots[r]) continue;
      a.slots[r][(size_t)i * a.blocks_per_item + jj] =
          live ? resolve_slot(h, a.map[r], a.n_handles, a.n_gpu_blocks, a.n_slots, a.stage_valid[r] != 0, a.err) : -1;
    }
  }
}

struct AttnArgs {
  const char* kv_layer;
  const int32_t* slots;      // per item: device slots of its blocks, for this layer's staging region
  const uint2* items;
  const int32_t* hdr;
  uint32_t* counter;         // ticket counter of this launch (zeroed by the planning kernel)
  const char* q;             // [B][Hq][d]
  char* out;                 // [B][Hq][d]
  float* ws;                 // [B][Hq][n_parts][2 + d]
  const int32_t* ctx;
  size_t block_bytes;
  float scale_log2e;
  int32_t max_blocks, n_kv_heads, part_tokens, n_parts;
#ifdef PIE_EXPERIMENT
  unsigned long long* dbg;   // per-unit timestamps
  int32_t dbg_cap;
#endif
};

template <typename E, int HD, int G, bool NT>
__global__ __launch_bounds__(kWaves * 64) __attribute__((amdgpu_waves_per_eu((G == 1 && Elem<E>::kVec == 8) ? 4 : 1, 8)))
void k_attn_decode(const AttnArgs a) {
  using EL = Elem<E>;
  constexpr int VEC = EL::kVec;
  constexpr int LPR = HD / VEC;
  constexpr int TPL = 64 / LPR;
  constexpr int NLD = kBlockTokens / TPL;
  constexpr int TILE_BYTES = kBlockTokens * HD * (16 / VEC);
  constexpr int NP = kWaves * TPL;
  constexpr int EB = 16 / VEC;                 // bytes per element
  static_assert(LPR >= 4 && LPR <= 64 && NLD >= 1, "unsupported head_dim / dtype");

  __shared__ uint32_t s_ticket;
  __shared__ float s_m[NP], s_l[NP];
  __shared__ float s_acc[NP][HD];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int rg = lane / LPR, c = lane % LPR;
  const int32_t n_q_heads = a.n_kv_heads * G;
  const uint32_t n_kv = (uint32_t)a.n_kv_heads;
  const uint32_t n_units = (uint32_t)a.hdr[0] * n_kv;
  const size_t v_off = a.block_bytes / 2;
  const int32_t bpi = a.part_tokens / kBlockTokens;               // blocks per item, <= 64 * kWaves
  const int32_t my_n = (bpi + kWaves - 1 - wave) / kWaves;        // blocks of an item this wave may own

  // Units are handed out by tickets.  A workgroup's first two are static (its index, and its index plus the
  // grid size); the rest come from an atomic counter.  The ticket for the unit after next is requested
  // behind a unit's stream, so the next unit is always known one unit ahead, its metadata is fetched while
  // the current unit is merged, and no load ever waits behind the contended counter.
  uint32_t unit = blockIdx.x;
  uint32_t next = gridDim.x + blockIdx.x;

  uint2 rec = make_uint2(0, 0);
  int32_t my_slot = -1;
  uint4 qraw[G];
  if (unit < n_units) {
    const uint32_t item = unit / n_kv;
    rec = a.items[item];
    if (lane < my_n) my_slot = a.slots[(size_t)item * bpi + wave + kWaves * lane];
    const int32_t b0 = (int32_t)(rec.x & 0xffffu), g0 = (int32_t)(unit % n_kv);
#pragma unroll
    for (int h = 0; h < G; ++h)
      qraw[h] = *reinterpret_cast<const uint4*>(a.q + (((size_t)b0 * n_q_heads + g0 * G + h) * HD + c * VEC) * EB);
  }

  while (unit < n_units) {                       // every workgroup ends on a ticket past the last unit
    uint2 rec_next = make_uint2(0, 0);
    if (next < n_units) rec_next = a.items[next / n_kv];          // consumed after the stream loop
#ifdef PIE_EXPERIMENT
    const unsigned long long t_entry = wall_clock64();
#endif
    const int32_t g = (int32_t)(unit % n_kv);
    const int32_t b = (int32_t)(rec.x & 0xffffu), part = (int32_t)(rec.x >> 16);
    const int32_t tok0 = part * a.part_tokens;
    const int32_t tok1 = (int32_t)rec.y;                           // <= tok0 only for an empty sequence
    const int32_t hq0 = g * G;

    // blocks of this item handled by this wave: j = jb0 + wave + kWaves * it
    const int32_t jb0 = tok0 / kBlockTokens;
    const int32_t jb1 = tok1 > 0 ? (tok1 + kBlockTokens - 1) / kBlockTokens : 0;   // exclusive, <= max_blocks
    const int32_t n_it = (jb1 - jb0 - wave + kWaves - 1) / kWaves;  // <= my_n <= 64; <= 0 when nothing to do

    // query rows of the G heads, this lane's VEC dims, as fp32 pre-multiplied by scale*log2(e)
    float q[G][VEC];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      EL::unpack(qraw[h], q[h]);
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

    const size_t head_off = (size_t)g * TILE_BYTES;

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
    // the ticket after next is requested half way through the stream: late enough that the counter is not
    // hit by every workgroup at once, early enough that the answer is there when the unit ends
    uint32_t after_next = 0;
    const int32_t it_ticket = n_it > 2 ? ((n_it / 2) & ~1) : 0;
    if (n_it > 0) load_tile(kA, vA, 0);
    for (int32_t it = 0; it < n_it; it += 2) {
      if (it == it_ticket && threadIdx.x == 0) after_next = 2 * gridDim.x + atomicAdd(a.counter, 1u);
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

    if (n_it <= 0 && threadIdx.x == 0) after_next = 2 * gridDim.x + atomicAdd(a.counter, 1u);
    // behind the stream: the next unit's slots and query rows arrive while this unit's result is merged
    int32_t my_slot_next = -1;
    if (next < n_units) {
      const uint32_t item_n = next / n_kv;
      if (lane < my_n) my_slot_next = a.slots[(size_t)item_n * bpi + wave + kWaves * lane];
      const int32_t bn = (int32_t)(rec_next.x & 0xffffu), gn = (int32_t)(next % n_kv);
#pragma unroll
      for (int h = 0; h < G; ++h)
        qraw[h] = *reinterpret_cast<const uint4*>(a.q + (((size_t)bn * n_q_heads + gn * G + h) * HD + c * VEC) * EB);
    }

    // merge the kWaves * TPL partial states, one query head at a time to keep LDS small
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
    if (threadIdx.x == 0) s_ticket = after_next;
#ifdef PIE_EXPERIMENT
    if (a.dbg && lane == 0 && (int32_t)unit < a.dbg_cap) {
      unsigned long long* d = a.dbg + ((size_t)unit * kWaves + wave) * 6;
      d[0] = t_entry; d[1] = t_pro; d[2] = t_loop; d[3] = wall_clock64();
      d[4] = (unsigned long long)(n_it > 0 ? n_it : 0);
      unsigned xcc; asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
      d[5] = ((unsigned long long)xcc << 32) | blockIdx.x;
    }
#endif
    __syncthreads();                             // merge buffers free again; the new ticket is visible
    unit = next;
    next = s_ticket;
    rec = rec_next;
    my_slot = my_slot_next;
    __syncthreads();                             // all have read the ticket before it is overwritten
  }
}

// Reduction over the partitions of one (sequence, query head): out = sum_s 2^(m_s - M) acc_s / sum_s 2^(m_s - M) l_s.
template <typename E, int HD>
__global__ __launch_bounds__(HD) void k_attn_reduce(const AttnArgs a, int32_t n_q_heads) {
  using EL = Elem<E>;
  const int32_t hq = blockIdx.x, b = blockIdx.y, dim = threadIdx.x;
  const int32_t ctx = clamp_ctx(a.ctx[b], a.max_blocks);
  int32_t np = ctx <= 0 ? 1 : (ctx + a.part_tokens - 1) / a.part_tokens;
  if (np > a.n_parts) np = a.n_parts;
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

static bool pick(int32_t dtype, int32_t hd, int32_t g) {
  if (dtype < 0 || dtype > 2) return false;
  if (hd != 64 && hd != 128) return false;
  return g == 1 || g == 2 || g == 4 || g == 8;
}

bool attn_config_supported(const pie_config& c) {
  return c.block_tokens == kBlockTokens && pick(c.dtype, c.head_dim, c.n_q_heads / c.n_kv_heads) &&
         c.max_batch <= kMaxPlanBatch && c.max_blocks_per_seq <= (1 << 19);
}

static size_t max_parts_of(const pie_config& c) {
  const size_t mp = ((size_t)c.max_blocks_per_seq * c.block_tokens + kMinPartTokens - 1) / kMinPartTokens;
  return mp ? mp : 1;
}

size_t attn_workspace_floats(const pie_config& c) {
  return (size_t)c.max_batch * c.n_q_heads * max_parts_of(c) * (c.head_dim + 2);
}

// Blocks of slot lists one region needs: every item lists part_tokens / 16 slots, and a sequence's items
// cover its blocks rounded up to a whole item.
static size_t slot_list_ints(const pie_config& c) {
  return (size_t)c.max_batch * ((size_t)c.max_blocks_per_seq + kWaves * 64);
}

// int32 words of planning state: header, per-layer ticket counters, item records (2 words each), and the
// per-item slot lists of the two staging regions
size_t attn_plan_ints(const pie_config& c) {
  return kPlanHdrInts + (size_t)c.n_layers + ((size_t)c.n_layers & 1) + 2 * (size_t)c.max_batch * max_parts_of(c) +
         2 * slot_list_ints(c);
}

static int32_t* plan_hdr(const pie_pool* p) { return p->d_plan; }
static uint32_t* plan_counters(const pie_pool* p) { return reinterpret_cast<uint32_t*>(p->d_plan + kPlanHdrInts); }
static size_t plan_items_off(const pie_pool* p) {          // kept 8-byte aligned
  return kPlanHdrInts + (size_t)p->cfg.n_layers + ((size_t)p->cfg.n_layers & 1);
}
static uint2* plan_items(const pie_pool* p) { return reinterpret_cast<uint2*>(p->d_plan + plan_items_off(p)); }
static int32_t* plan_slots(const pie_pool* p, int region) {
  return p->d_plan + plan_items_off(p) + 2 * (size_t)p->cfg.max_batch * max_parts_of(p->cfg) +
         (size_t)region * slot_list_ints(p->cfg);
}

// item size: a multiple of one pass of the workgroup's waves, at most 64 blocks per wave
static int32_t part_tokens_of(const pie_pool* p) {
  int32_t part = p->attn_partition;
  const int32_t quantum = kWaves * kBlockTokens;
  if (part < kMinPartTokens) part = kMinPartTokens;
  part = (part + quantum - 1) / quantum * quantum;
  if (part > quantum * 64) part = quantum * 64;
  return part;
}

int launch_attn_plan(const pie_pool* p, const int32_t* d_ctx, int32_t batch, int32_t max_blocks, hipStream_t s) {
  if (batch > kMaxPlanBatch || batch > p->cfg.max_batch || max_blocks > p->cfg.max_blocks_per_seq) return PIE_EINVAL;
  hipLaunchKernelGGL(k_attn_plan, dim3(1), dim3(256), 0, s, d_ctx, batch, part_tokens_of(p), max_blocks, plan_items(p),
                     plan_hdr(p), plan_counters(p), p->cfg.n_layers, p->d_err);
  PIE_HIP(hipGetLastError());
  return PIE_OK;
}

int launch_attn_resolve(const pie_pool* p, const int32_t* d_table, const int32_t* d_ctx, int32_t batch,
                        int32_t max_blocks, bool region0, bool valid0, bool region1, bool valid1, hipStream_t s) {
  (void)d_ctx;
  if (batch > p->cfg.max_batch || max_blocks > p->cfg.max_blocks_per_seq || max_blocks <= 0) return PIE_EINVAL;
  const int32_t part = part_tokens_of(p);
  ResolveArgs a;
  a.table = d_table;
  a.items = plan_items(p);
  a.hdr = plan_hdr(p);
  a.map[0] = p->d_map[0];
  a.map[1] = p->d_map[1];
  a.slots[0] = region0 ? plan_slots(p, 0) : nullptr;
  a.slots[1] = region1 ? plan_slots(p, 1) : nullptr;
  a.err = p->d_err;
  a.max_blocks = max_blocks;
  a.n_handles = p->n_handles;
  a.n_gpu_blocks = p->cfg.n_gpu_blocks;
  a.n_slots = p->cfg.n_gpu_blocks + 2 * p->cfg.n_stage_blocks;
  a.blocks_per_item = part / kBlockTokens;
  a.stage_valid[0] = valid0 ? 1 : 0;
  a.stage_valid[1] = valid1 ? 1 : 0;
  // one workgroup per possible item; those past the planned count return at once
  const int32_t max_items = batch * ((max_blocks * kBlockTokens + part - 1) / part);
  hipLaunchKernelGGL(k_attn_resolve, dim3(max_items), dim3(64), 0, s, a);
  PIE_HIP(hipGetLastError());
  return PIE_OK;
}

template <typename E, int HD, int G>
static int launch_typed(const pie_pool* p, const AttnArgs& a, int32_t batch, int32_t n_q_heads, hipStream_t s,
                        hipEvent_t e0, hipEvent_t e1) {
  // as many workgroups as fit on the GPU at once; the ticket counter hands out the work
  static int wgs_per_cu = 0;
  if (wgs_per_cu == 0) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_attn_decode<E, HD, G, true>, kWaves * 64, 0) != hipSuccess || n < 1) {
      (void)hipGetLastError();
      n = 2;
    }
    wgs_per_cu = n;
  }
  const int grid = p->n_cu * wgs_per_cu;
  if (e0) PIE_HIP(hipEventRecord(e0, s));
  if (p->attn_nontemporal)
    hipLaunchKernelGGL((k_attn_decode<E, HD, G, true>), dim3(grid), dim3(kWaves * 64), 0, s, a);
  else
    hipLaunchKernelGGL((k_attn_decode<E, HD, G, false>), dim3(grid), dim3(kWaves * 64), 0, s, a);
  PIE_HIP(hipGetLastError());
  if (e1) PIE_HIP(hipEventRecord(e1, s));
  if (a.n_parts > 1) {
    hipLaunchKernelGGL((k_attn_reduce<E, HD>), dim3(n_q_heads, batch), dim3(HD), 0, s, a, n_q_heads);
    PIE_HIP(hipGetLastError());
  }
  return PIE_OK;
}

template <typename E, int HD>
static int launch_g(const pie_pool* p, const AttnArgs& a, int32_t g, int32_t batch, int32_t nq, hipStream_t s,
                    hipEvent_t e0, hipEvent_t e1) {
  switch (g) {
    case 1: return launch_typed<E, HD, 1>(p, a, batch, nq, s, e0, e1);
    case 2: return launch_typed<E, HD, 2>(p, a, batch, nq, s, e0, e1);
    case 4: return launch_typed<E, HD, 4>(p, a, batch, nq, s, e0, e1);
    case 8: return launch_typed<E, HD, 8>(p, a, batch, nq, s, e0, e1);
    default: return PIE_EINVAL;
  }
}

template <typename E>
static int launch_hd(const pie_pool* p, const AttnArgs& a, int32_t hd, int32_t g, int32_t batch, int32_t nq,
                     hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  switch (hd) {
    case 64: return launch_g<E, 64>(p, a, g, batch, nq, s, e0, e1);
    case 128: return launch_g<E, 128>(p, a, g, batch, nq, s, e0, e1);
    default: return PIE_EINVAL;
  }
}

// Needs launch_attn_plan and launch_attn_resolve (for region layer & 1) earlier on the same stream, with the
// same batch, table width and context lengths.
int launch_attn_decode(const pie_pool* p, int32_t layer, const void* d_q, int32_t max_blocks, const int32_t* d_ctx,
                       int32_t batch, void* d_out, hipStream_t s, hipEvent_t k_start, hipEvent_t k_end) {
  const pie_config& c = p->cfg;
  if (((uintptr_t)d_q | (uintptr_t)d_out) % 16) return PIE_EINVAL;
  if (max_blocks <= 0) return PIE_EINVAL;
  if (c.n_gpu_blocks + 2 * c.n_stage_blocks <= 0) return PIE_EINVAL;
  const int32_t g = c.n_q_heads / c.n_kv_heads;
  const int32_t part = part_tokens_of(p);
  const int32_t max_tokens = max_blocks * kBlockTokens;
  const int32_t n_parts = (max_tokens + part - 1) / part;
  if ((size_t)batch * c.n_q_heads * n_parts * (c.head_dim + 2) > p->ws_floats) return PIE_ENOMEM;

  AttnArgs a;
  a.kv_layer = p->d_kv + (size_t)layer * p->d_layer_stride;
  a.slots = plan_slots(p, layer & 1);
  a.items = plan_items(p);
  a.hdr = plan_hdr(p);
  a.counter = plan_counters(p) + layer;
  a.q = (const char*)d_q;
  a.out = (char*)d_out;
  a.ws = p->d_ws;
  a.ctx = d_ctx;
  a.block_bytes = p->block_bytes;
  a.scale_log2e = p->scale_log2e;
  a.max_blocks = max_blocks;
  a.n_kv_heads = c.n_kv_heads;
  a.part_tokens = part;
  a.n_parts = n_parts;
#ifdef PIE_EXPERIMENT
  { const char* e = getenv("PIE_DBG_PTR"); a.dbg = e ? (unsigned long long*)strtoull(e, nullptr, 10) : nullptr;
    const char* c2 = getenv("PIE_DBG_CAP"); a.dbg_cap = c2 ? atoi(c2) : 0; }
#endif
  switch (c.dtype) {
    case PIE_DTYPE_F32: return launch_hd<F32>(p, a, c.head_dim, g, batch, c.n_q_heads, s, k_start, k_end);
    case PIE_DTYPE_F16: return launch_hd<F16>(p, a, c.head_dim, g, batch, c.n_q_heads, s, k_start, k_end);
    case PIE_DTYPE_BF16: return launch_hd<BF16>(p, a, c.head_dim, g, batch, c.n_q_heads, s, k_start, k_end);
    default: return PIE_EINVAL;
  }
}

}  // namespace pie
