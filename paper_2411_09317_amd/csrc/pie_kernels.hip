// HIP kernels for gfx950 (CDNA4, 64-wide wavefronts): paged-attention decode with a split over the
// context and its reduction, the KV append, the block gather / scatter used by swaps, and the small
// map-maintenance kernels.
//
// What the attention kernels compute is the paged KV-cache attention of the paper's Section 2.3 for the
// per-layer access pattern of Section 3.2:
//   out[b][h] = sum_t softmax_t(scale * <q[b][h], K[b][g][t]>) V[b][g][t],   t < ctx_b,  g = h / (Hq/Hkv).
//
// One block of one layer holds the K tiles of the kv heads, then their V tiles; inside a tile the elements are
// ordered so that a 16-byte lane vector is a matrix-core operand as loaded (see "element types and the layout
// of a block" below).  The decode is bound by HBM bandwidth: every KV byte of the layer is read exactly once,
// with 16-byte loads per lane that cover a tile in contiguous 1 KiB pieces.

#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <mutex>

#include <hip/hip_ext.h>

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

// Occupies a stream for about `ticks` ticks of the constant wall clock: one wave that sleeps and looks at
// the clock.  max_iter bounds the loop, so the wave exits whatever the clock does.
__global__ void k_busy(unsigned long long ticks, uint32_t max_iter, unsigned long long* clock) {
  const unsigned long long t0 = wall_clock64();
  for (uint32_t i = 0; i < max_iter; ++i) {
    if (wall_clock64() - t0 >= ticks) break;
    __builtin_amdgcn_s_sleep(16);
  }
  if (clock && threadIdx.x == 0) atomicMax(&clock[kClockLayerEnd], wall_clock64());
}

// ---- device-clock time stamps ---------------------------------------------------------------------------
// With monitoring by device clock a layer's kernels note when they ran, read from the constant-rate wall
// clock all compute units share; nothing is recorded between kernels, so they stay back to back.  Each layer
// has a row of 64-bit words (kClock*).  Atomics on one address cost about 8 ns each and all of it shows in
// the kernel's duration, so the persistent decode kernel's workgroups write their first and last moment to
// words of their own (kClockWgs pairs per layer) and k_clock_fold, once per step, folds them into the row;
// kernels with few workgroups, or few that matter, use atomic min / max on the row directly.  Work on the
// swap streams is bracketed by k_stamp.
__global__ void k_stamp(unsigned long long* slot) {
  if (threadIdx.x == 0) *slot = wall_clock64();
}

// One workgroup per layer: row[KernelStart / KernelEnd] take in the per-workgroup pairs (row[kClockGrid] of
// them), and row[LayerEnd] is at least the kernel's end.
__global__ __launch_bounds__(256) void k_clock_fold(unsigned long long* __restrict__ rows,
                                                    const unsigned long long* __restrict__ per_wg) {
  __shared__ unsigned long long s_lo[256], s_hi[256];
  unsigned long long* row = rows + (size_t)blockIdx.x * kClockRow;
  const unsigned long long* wg = per_wg + (size_t)blockIdx.x * kClockWgs * 2;
  unsigned long long n = row[kClockGrid];
  n = n > (unsigned long long)kClockWgs ? (unsigned long long)kClockWgs : n;
  unsigned long long lo = ~0ull, hi = 0ull;
  for (unsigned long long i = threadIdx.x; i < n; i += 256) {
    const unsigned long long a = wg[2 * i], b = wg[2 * i + 1];
    lo = a < lo ? a : lo;
    hi = b > hi ? b : hi;
  }
  s_lo[threadIdx.x] = lo;
  s_hi[threadIdx.x] = hi;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) {
      s_lo[threadIdx.x] = s_lo[threadIdx.x + w] < s_lo[threadIdx.x] ? s_lo[threadIdx.x + w] : s_lo[threadIdx.x];
      s_hi[threadIdx.x] = s_hi[threadIdx.x + w] > s_hi[threadIdx.x] ? s_hi[threadIdx.x + w] : s_hi[threadIdx.x];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const unsigned long long ks = row[kClockKernelStart], ke = row[kClockKernelEnd], le = row[kClockLayerEnd];
    const unsigned long long start = s_lo[0] < ks ? s_lo[0] : ks, end = s_hi[0] > ke ? s_hi[0] : ke;
    row[kClockKernelStart] = start;
    row[kClockKernelEnd] = end;
    row[kClockLayerEnd] = le > end ? le : end;
  }
}

int launch_clock_fold(unsigned long long* rows, int32_t n_layers, hipStream_t s) {
  hipLaunchKernelGGL(k_clock_fold, dim3(n_layers), dim3(256), 0, s, rows,
                     rows + ((size_t)n_layers + 1) * kClockRow);
  PIE_HIP(hipGetLastError());
  return PIE_OK;
}

int launch_stamp(unsigned long long* slot, hipStream_t s) {
  hipLaunchKernelGGL(k_stamp, dim3(1), dim3(64), 0, s, slot);
  PIE_HIP(hipGetLastError());
  return PIE_OK;
}

int launch_busy(double us, int wall_clock_khz, hipStream_t s, unsigned long long* clock, hipEvent_t done) {
  if (!(us > 0.0)) return PIE_OK;
  const unsigned long long ticks = (unsigned long long)(us * 1e-3 * (double)wall_clock_khz);
  // an iteration takes at least the sleep's 16 x 64 clocks, i.e. well over 0.1 us: 16 iterations per us plus
  // slack always reach the deadline first
  const uint32_t max_iter = (uint32_t)(us * 16.0) + 4096u;
  // `done` completes with the kernel itself: no separate packet on the stream
  if (done) hipExtLaunchKernelGGL(k_busy, dim3(1), dim3(64), 0, s, nullptr, done, 0, ticks, max_iter, clock);
  else hipLaunchKernelGGL(k_busy, dim3(1), dim3(64), 0, s, ticks, max_iter, clock);
  PIE_HIP(hipGetLastError());
  return PIE_OK;
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

// A layer whose blocks are spread over chunks of `chunk_blocks` consecutive slots: block h lives in slot
// chunks[h / chunk_blocks] * chunk_blocks + h % chunk_blocks; blocks beyond the layer's chunks map to -1.
__global__ void k_chunk_map_fill(int32_t* __restrict__ map, int32_t n_handles, int32_t chunk_blocks, const ChunkList list) {
  const int32_t h = blockIdx.x * blockDim.x + threadIdx.x;
  if (h >= n_handles) return;
  const int32_t c = h / chunk_blocks;
  map[h] = c < list.n ? list.chunk[c] * chunk_blocks + h % chunk_blocks : -1;
}

int launch_chunk_map_fill(int32_t* d_map, int32_t n_handles, int32_t chunk_blocks, const ChunkList& list, hipStream_t s) {
  if (n_handles <= 0) return PIE_OK;
  hipLaunchKernelGGL(k_chunk_map_fill, dim3((n_handles + 255) / 256), dim3(256), 0, s, d_map, n_handles, chunk_blocks, list);
  PIE_HIP(hipGetLastError());
  return PIE_OK;
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
// the host link: what matters is the number of 16-byte requests in flight, not the number of CUs (one compute
// unit sustains about 3.5 GB/s per wavefront with sixteen loads in flight, at most about 14 GB/s).  A fixed,
// small grid strides over pieces of THREADS x UNROLL 16-byte vectors; each lane keeps UNROLL loads in flight.
// ---------------------------------------------------------------------------------------------------

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int THREADS, int UNROLL>
__global__ __launch_bounds__(THREADS) void k_swap_copy(char* __restrict__ dst_base, const char* __restrict__ src_base,
                                                       size_t block_bytes, const SwapPairs pairs) {
  constexpr size_t kPiece = (size_t)THREADS * 16 * UNROLL;        // bytes per workgroup iteration
  // few instructions, long waits: let them issue ahead of the decode kernel's waves on the same compute unit
  __builtin_amdgcn_s_setprio(3);
  const size_t pieces_per_block = (block_bytes + kPiece - 1) / kPiece;
  const size_t n_pieces = pieces_per_block * (size_t)pairs.n;
  for (size_t piece = blockIdx.x; piece < n_pieces; piece += gridDim.x) {
    const int32_t i = (int32_t)(piece / pieces_per_block);
    const size_t off = (piece % pieces_per_block) * kPiece;
    const u32x4* s = reinterpret_cast<const u32x4*>(src_base + (size_t)pairs.src[i] * block_bytes + off);
    u32x4* d = reinterpret_cast<u32x4*>(dst_base + (size_t)pairs.dst[i] * block_bytes + off);
    const size_t n16 = (block_bytes - off < kPiece ? block_bytes - off : kPiece) / 16;
    u32x4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const size_t j = (size_t)u * THREADS + threadIdx.x;
      if (j < n16) v[u] = __builtin_nontemporal_load(s + j);
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const size_t j = (size_t)u * THREADS + threadIdx.x;
      if (j < n16) __builtin_nontemporal_store(v[u], d + j);
    }
  }
}

template <int THREADS, int UNROLL>
static int launch_swap_copy_as(char* dst_layer_base, const char* src_layer_base, size_t block_bytes,
                               const SwapPairs& pairs, int n_wgs, hipStream_t s) {
  constexpr size_t kPiece = (size_t)THREADS * 16 * UNROLL;
  const size_t pieces = ((block_bytes + kPiece - 1) / kPiece) * (size_t)pairs.n;
  const int grid = (int)(pieces < (size_t)n_wgs ? pieces : (size_t)n_wgs);
  hipLaunchKernelGGL((k_swap_copy<THREADS, UNROLL>), dim3(grid), dim3(THREADS), 0, s, dst_layer_base, src_layer_base,
                     block_bytes, pairs);
  PIE_HIP(hipGetLastError());
  return PIE_OK;
}

// shape: threads per workgroup x 16-byte loads in flight per lane, as threads * 100 + loads; 0 = chosen here
// from the size of the transfer.  What was measured beside the decode kernel of the 7B-shaped workload
// (265 us per layer, every compute unit streaming from HBM):
//  - While the decode kernel runs, a gather wave's requests queue behind the decode waves' in the compute
//    unit's memory pipeline and the link rate is set by the number of gather waves, whatever each has in
//    flight: 64 waves move about 28 GB/s, 128 about 45 GB/s; the decode kernel slows by 2-3 %.
//  - A gather that outlasts the layer runs alone part of the time and then reaches 40-55 GB/s with few waves,
//    but at full speed it costs the decode kernel next to it more: workgroups of 256 threads, 8 / 16 / 64 of
//    them: +4-5 % / +15 % / +110 %; one-wave workgroups with sixteen loads in flight, which fit beside the
//    decode kernel's resident workgroups instead of displacing one, 12 / 16 of them: +1-2 % / +2-3 % at
//    39 / 41 GB/s.
// So a transfer small enough to hide behind a layer is moved by n_wgs workgroups of 256 threads (it must finish
// before the layer does), and a larger one, for which the layer will wait in any case, by n_wgs one-wave
// workgroups (it must not slow the layers it runs beside).
constexpr size_t kGatherSmallBytes = (size_t)12 << 20;

int launch_swap_copy(char* dst_layer_base, const char* src_layer_base, size_t block_bytes, const SwapPairs& pairs,
                     int n_wgs, hipStream_t s, int shape, size_t transfer_bytes) {
  if (pairs.n <= 0) return PIE_OK;
  if (block_bytes % 16 || n_wgs < 1) return PIE_EINVAL;
  if (shape == 0) shape = (transfer_bytes ? transfer_bytes : block_bytes * pairs.n) <= kGatherSmallBytes ? 25604 : 6416;
  switch (shape) {
    case 6404: return launch_swap_copy_as<64, 4>(dst_layer_base, src_layer_base, block_bytes, pairs, n_wgs, s);
    case 6416: return launch_swap_copy_as<64, 16>(dst_layer_base, src_layer_base, block_bytes, pairs, n_wgs, s);
    case 25602: return launch_swap_copy_as<256, 2>(dst_layer_base, src_layer_base, block_bytes, pairs, n_wgs, s);
    case 25604: return launch_swap_copy_as<256, 4>(dst_layer_base, src_layer_base, block_bytes, pairs, n_wgs, s);
    case 102416: return launch_swap_copy_as<1024, 16>(dst_layer_base, src_layer_base, block_bytes, pairs, n_wgs, s);
    default: return PIE_EINVAL;
  }
}

// ---------------------------------------------------------------------------------------------------
// element types and the layout of a block
//
// A block is [K tiles of the kv heads][V tiles of the kv heads]; a tile is 16 tokens x head_dim elements.
// With v = 16 / elem_bytes elements per 16-byte vector and w = v / 4:
//   K tile: element (token t, dim c) at  (c / v) * (16 v) + t v + c % v
//           -> a vector holds v consecutive dims of one token; lane i of a 64-lane load of 1 KiB gets
//              token i % 16, dims 8 (i / 16) .. of a 4-vector-wide slab: the A operand of a 16x16x32 MFMA.
//   V tile: element (t, c) at  (((c / (16 w)) * 4 + t / 4) * 16 + c % 16) * v + ((c / 16) % w) * 4 + t % 4
//           -> a vector holds 4 consecutive tokens of dim c (and, 16-bit, of dim c + 16); lane i of a 1 KiB
//              load gets tokens 4 (i / 16) .., dim i % 16 of a 16 w-dim slab: the A operand(s) of 16x16x16 MFMAs
//              whose contraction runs over the 16 tokens of the block.
// ---------------------------------------------------------------------------------------------------

struct F32 { static constexpr int kBytes = 4; };
struct F16 { static constexpr int kBytes = 2; };
struct BF16 { static constexpr int kBytes = 2; };

__host__ __device__ __forceinline__ int32_t k_tile_index(int32_t t, int32_t c, int32_t v) {
  return (c / v) * (16 * v) + t * v + c % v;
}
__host__ __device__ __forceinline__ int32_t v_tile_index(int32_t t, int32_t c, int32_t v) {
  const int32_t w = v / 4;
  return (((c / (16 * w)) * 4 + t / 4) * 16 + c % 16) * v + ((c / 16) % w) * 4 + t % 4;
}

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);                                            // nearest even
  return (uint16_t)(u >> 16);
}

template <typename E> __device__ __forceinline__ float load_elem(const void* base, size_t idx);
template <> __device__ __forceinline__ float load_elem<F32>(const void* base, size_t idx) {
  return reinterpret_cast<const float*>(base)[idx];
}
template <> __device__ __forceinline__ float load_elem<F16>(const void* base, size_t idx) {
  return __half2float(reinterpret_cast<const __half*>(base)[idx]);
}
template <> __device__ __forceinline__ float load_elem<BF16>(const void* base, size_t idx) {
  return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(base)[idx] << 16);
}

// two consecutive elements, idx even
template <typename E> __device__ __forceinline__ float2 load_elem2(const void* base, size_t idx);
template <> __device__ __forceinline__ float2 load_elem2<F32>(const void* base, size_t idx) {
  return *reinterpret_cast<const float2*>(reinterpret_cast<const float*>(base) + idx);
}
template <> __device__ __forceinline__ float2 load_elem2<F16>(const void* base, size_t idx) {
  return __half22float2(*reinterpret_cast<const __half2*>(reinterpret_cast<const __half*>(base) + idx));
}
template <> __device__ __forceinline__ float2 load_elem2<BF16>(const void* base, size_t idx) {
  const uint32_t u = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const uint16_t*>(base) + idx);
  return make_float2(__uint_as_float(u << 16), __uint_as_float(u & 0xffff0000u));
}

template <typename E> __device__ __forceinline__ void store_elem(void* base, size_t idx, float v);
template <> __device__ __forceinline__ void store_elem<F32>(void* base, size_t idx, float v) {
  reinterpret_cast<float*>(base)[idx] = v;
}
template <> __device__ __forceinline__ void store_elem<F16>(void* base, size_t idx, float v) {
  reinterpret_cast<__half*>(base)[idx] = __float2half_rn(v);
}
template <> __device__ __forceinline__ void store_elem<BF16>(void* base, size_t idx, float v) {
  reinterpret_cast<uint16_t*>(base)[idx] = f32_to_bf16_bits(v);
}

template <typename E> __device__ __forceinline__ void store_elem2(void* base, size_t idx, float2 v);
template <> __device__ __forceinline__ void store_elem2<F32>(void* base, size_t idx, float2 v) {
  *reinterpret_cast<float2*>(reinterpret_cast<float*>(base) + idx) = v;
}
template <> __device__ __forceinline__ void store_elem2<F16>(void* base, size_t idx, float2 v) {
  *reinterpret_cast<__half2*>(reinterpret_cast<__half*>(base) + idx) = __floats2half2_rn(v.x, v.y);
}
template <> __device__ __forceinline__ void store_elem2<BF16>(void* base, size_t idx, float2 v) {
  *reinterpret_cast<uint32_t*>(reinterpret_cast<uint16_t*>(base) + idx) =
      (uint32_t)f32_to_bf16_bits(v.x) | ((uint32_t)f32_to_bf16_bits(v.y) << 16);
}

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

constexpr int kAppendBlockTokens = 16;

struct AppendArgs {
  char* kv_layer;            // device pool base of this layer
  const int32_t* map;
  uint32_t* err;
  const char* k_new;         // [B][Hkv][d]
  const char* v_new;
  const int32_t* table;
  const int32_t* ctx;
  size_t block_bytes;
  size_t kv_layer_stride;    // blockIdx.y walks layers: bytes between layers in the pool ...
  size_t new_layer_stride;   // ... and in k_new / v_new
  int32_t max_blocks, n_handles, n_gpu_blocks, n_slots, n_kv_heads, head_dim, block_tokens, elem_bytes;
  int32_t mode;              // kAppend*: which tail blocks this launch writes
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
  if (threadIdx.x == 0) {
    int32_t slot = -1;
    const int32_t handle = a.table[(size_t)b * a.max_blocks + j];
    if (handle < 0 || handle >= a.n_handles) {
      atomicOr(a.err, PIE_DEVERR_BAD_HANDLE);
    } else {
      slot = a.map[handle];
      const bool gpu_homed = slot >= 0 && slot < a.n_gpu_blocks;
      const bool staged = slot >= a.n_gpu_blocks && slot < a.n_slots;
      bool take = false, missing = false;
      switch (a.mode) {
        case kAppendPresent: take = gpu_homed || staged; missing = !take; break;
        case kAppendGpuStrict: take = gpu_homed; missing = !take; break;
        case kAppendGpuHomed: take = gpu_homed; missing = !gpu_homed && !staged && slot != -1; break;
        default: take = staged; missing = !gpu_homed && !staged; break;                    // kAppendStaged
      }
      if (missing) atomicOr(a.err, PIE_DEVERR_NOT_PRESENT);
      if (!take) slot = -1;
    }
    s_slot = slot;
  }
  __syncthreads();
  const int32_t slot = s_slot;
  if (slot < 0) return;
  // one 16-byte vector of a key row goes to one vector of the K tile; a value row is scattered element by
  // element over the V tile's token-quad vectors
  const int32_t v = 16 / a.elem_bytes;
  const int32_t vec_per_row = a.head_dim / v;
  const int32_t tile_bytes = kAppendBlockTokens * a.head_dim * a.elem_bytes;
  char* blk = a.kv_layer + blockIdx.y * a.kv_layer_stride + (size_t)slot * a.block_bytes;
  const char* k_new = a.k_new + blockIdx.y * a.new_layer_stride;
  const char* v_new = a.v_new + blockIdx.y * a.new_layer_stride;
  const size_t v_off = a.block_bytes / 2;
  const int32_t t = pos % kAppendBlockTokens;
  const int32_t n_vec = a.n_kv_heads * vec_per_row;
  for (int32_t i = threadIdx.x; i < n_vec; i += blockDim.x) {
    const int32_t g = i / vec_per_row, cv = i % vec_per_row;
    const size_t src = ((size_t)b * a.n_kv_heads + g) * a.head_dim * a.elem_bytes + (size_t)cv * 16;
    const size_t dst = (size_t)g * tile_bytes + (size_t)k_tile_index(t, cv * v, v) * a.elem_bytes;
    *reinterpret_cast<uint4*>(blk + dst) = *reinterpret_cast<const uint4*>(k_new + src);
  }
  const int32_t n_el = a.n_kv_heads * a.head_dim;
  for (int32_t i = threadIdx.x; i < n_el; i += blockDim.x) {
    const int32_t g = i / a.head_dim, c = i % a.head_dim;
    const size_t src = ((size_t)b * a.n_kv_heads + g) * a.head_dim + c;
    const size_t dst = v_off + (size_t)g * tile_bytes + (size_t)v_tile_index(t, c, v) * a.elem_bytes;
    if (a.elem_bytes == 2)
      *reinterpret_cast<uint16_t*>(blk + dst) = reinterpret_cast<const uint16_t*>(v_new)[src];
    else
      *reinterpret_cast<uint32_t*>(blk + dst) = reinterpret_cast<const uint32_t*>(v_new)[src];
  }
}

// Appends for n_layers consecutive layers starting at `layer` in one launch.  With n_layers > 1 only modes
// that leave staged copies alone make sense (staging regions hold one layer each).
int launch_kv_append(const pie_pool* p, int32_t layer, int32_t n_layers, const void* d_k, const void* d_v,
                     const int32_t* d_table, int32_t max_blocks, const int32_t* d_ctx, int32_t batch,
                     int32_t mode, hipStream_t s, const LayerView* view) {
  if (((uintptr_t)d_k | (uintptr_t)d_v) % 16) return PIE_EINVAL;
  if (n_layers < 1 || (n_layers > 1 && (mode == kAppendPresent || mode == kAppendStaged))) return PIE_EINVAL;
  if (view && n_layers != 1) return PIE_EINVAL;
  AppendArgs a;
  a.kv_layer = p->d_kv + (size_t)layer * p->d_layer_stride;
  a.map = p->d_map[layer & 1];
  a.err = p->d_err;
  a.k_new = (const char*)d_k;
  a.v_new = (const char*)d_v;
  a.table = d_table;
  a.ctx = d_ctx;
  a.block_bytes = p->block_bytes;
  a.kv_layer_stride = p->d_layer_stride;
  a.new_layer_stride = (size_t)batch * p->cfg.n_kv_heads * p->cfg.head_dim * p->elem_bytes;
  a.max_blocks = max_blocks;
  a.n_handles = p->n_handles;
  a.n_gpu_blocks = p->cfg.n_gpu_blocks;
  a.n_slots = p->cfg.n_gpu_blocks + 2 * p->cfg.n_stage_blocks;
  a.n_kv_heads = p->cfg.n_kv_heads;
  a.head_dim = p->cfg.head_dim;
  a.block_tokens = p->cfg.block_tokens;
  a.elem_bytes = p->elem_bytes;
  a.mode = mode;
  if (view) {                                    // the layer's blocks live elsewhere: all of them "GPU-homed" there
    a.kv_layer = view->kv_base;
    a.map = view->map;
    a.n_handles = view->n_handles;
    a.n_gpu_blocks = a.n_slots = view->n_slots;
  }
  hipLaunchKernelGGL(k_kv_append, dim3(batch, n_layers), dim3(256), 0, s, a);
  PIE_HIP(hipGetLastError());
  return PIE_OK;
}

// ---------------------------------------------------------------------------------------------------
// paged-attention decode
//
// Work is cut into items: `part_tokens` consecutive tokens of one sequence.  A small planning kernel lists
// the non-empty items, full ones first and the sequences' shorter last pieces after them in descending
// size, and a resolve kernel turns the block table (handles) into device slots once per step.
//
// 16-bit caches (fp16 / bf16): k_attn_decode_mfma.  The kernel is persistent: about as many workgroups as
// the GPU can hold resident, each taking (item, kv head) units from an atomic ticket counter until none are
// left.  That evens out the 8 XCDs (which do not stream at the same rate), leaves only small units for the
// end of the launch, and pays the launch ramp once.  A workgroup of kWaves wavefronts handles one unit and
// all G <= 16 query heads that share the kv head; wave w takes blocks w, w + kWaves, ... of the item.
// Per block a wave issues head_dim/32 K loads and head_dim/32 V loads of 16 bytes per lane, each covering
// 1 KiB contiguous, non-temporal (every KV byte is read once), double-buffered in registers.  The loaded
// vectors are matrix-core operands as they are:
//   S[token][head]  = sum_c K[token][c] Q[head][c]      head_dim/32 x  v_mfma_f32_16x16x32   (A = K, B = Q)
//   O[dim][head]   += sum_t V[t][dim] P[t][head]        head_dim/16 x  v_mfma_f32_16x16x16   (A = V, B = P)
// The 16 columns are the query heads of the group (columns >= G carry zeros); for G = 1 the products are
// matrix-vector and most of the matrix core idles, which costs nothing: the kernel is bound by HBM, and what
// the matrix core buys is that no vector-ALU work is spent on unpacking and multiplying the 16-bit elements.
// The accumulator layout of S (lane = 16 (token / 4) + head, register = token % 4) is the B-operand layout
// of the 16x16x16 form, so P goes from the softmax into the second product without leaving its lane.
// The softmax is online, in the log2 domain, with one running maximum per head shared by the wave (two
// cross-lane swaps per block); the accumulators are rescaled only when some maximum moved.  P is rounded
// to the cache's 16-bit type for the second product; for bf16 the rounding residue goes through a second
// MFMA so that P carries 16 significant bits.  At the end the kWaves partial states merge through LDS and
// are written out (single partition) or stored as (m, l, acc) for the reduction kernel.
//
// fp32 caches: k_attn_decode_f32, a plain vector-ALU kernel over the same items, one workgroup per
// (item, query head).  It exists for the fp32 parity configuration, which is latency-bound.
// ---------------------------------------------------------------------------------------------------

constexpr int kWaves = 4;
constexpr int kBlockTokens = 16;
constexpr int kMinPartTokens = 256;
constexpr int kMaxPlanBatch = 4096;   // sequences the planning kernel keeps in LDS
constexpr int kPlanHdrInts = 16;
constexpr int kMaxGroup = 16;         // query heads per kv head the MFMA kernel handles (its 16 columns)
constexpr float kNegBig = -1.0e30f;   // finite stand-in for -inf as the initial running max

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

template <typename TO, typename FROM>
__device__ __forceinline__ TO bits_as(const FROM& x) {
  static_assert(sizeof(TO) == sizeof(FROM), "size mismatch");
  TO y;
  __builtin_memcpy(&y, &x, sizeof(TO));
  return y;
}

template <typename E> struct Mfma;
template <> struct Mfma<F16> {
  __device__ static f32x4 qk(const uint4& a, const uint4& b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(bits_as<f16x8>(a), bits_as<f16x8>(b), c, 0, 0, 0);
  }
  __device__ static f32x4 pv(const uint2& a, const uint2& b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x16f16(bits_as<f16x4>(a), bits_as<f16x4>(b), c, 0, 0, 0);
  }
  __device__ static uint2 round(const f32x4& p) { return bits_as<uint2>(__builtin_convertvector(p, f16x4)); }
  __device__ static f32x4 widen(const uint2& r) { return __builtin_convertvector(bits_as<f16x4>(r), f32x4); }
};
template <> struct Mfma<BF16> {
  __device__ static f32x4 qk(const uint4& a, const uint4& b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(bits_as<bf16x8>(a), bits_as<bf16x8>(b), c, 0, 0, 0);
  }
  __device__ static f32x4 pv(const uint2& a, const uint2& b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(bits_as<s16x4>(a), bits_as<s16x4>(b), c, 0, 0, 0);
  }
  __device__ static uint2 round(const f32x4& p) { return bits_as<uint2>(__builtin_convertvector(p, bf16x4)); }
  __device__ static f32x4 widen(const uint2& r) {
    f32x4 f;
    f[0] = __uint_as_float(r.x << 16);
    f[1] = __uint_as_float(r.x & 0xffff0000u);
    f[2] = __uint_as_float(r.y << 16);
    f[3] = __uint_as_float(r.y & 0xffff0000u);
    return f;
  }
};

// Two-element dot products on the vector ALU (v_dot2_f32_f16 / v_dot2_f32_bf16): c + a.x b.x + a.y b.y with the
// products and the sum in fp32.  Used by the variant of the decode kernel that keeps off the matrix cores.
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
template <typename E> struct Dot2;
template <> struct Dot2<F16> {
  __device__ static float fma2(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2(bits_as<f16x2>(a), bits_as<f16x2>(b), c, false);
  }
};
template <> struct Dot2<BF16> {
  __device__ static float fma2(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(bits_as<bf16x2>(a), bits_as<bf16x2>(b), c, false);
  }
};

// max / sum over the four lanes i, i ^ 16, i ^ 32, i ^ 48; every lane gets the result
__device__ __forceinline__ float quad16_max(float x) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float quad16_sum(float x) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// max / sum over the 16 lanes of a row (lanes 16 r .. 16 r + 15); every lane of the row gets the result
template <int CTRL>
__device__ __forceinline__ float dpp_get(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float row16_max(float x) {
  x = fmaxf(x, dpp_get<0xB1>(x));    // quad_perm [1,0,3,2]: lane ^ 1
  x = fmaxf(x, dpp_get<0x4E>(x));    // quad_perm [2,3,0,1]: lane ^ 2
  x = fmaxf(x, dpp_get<0x141>(x));   // row_half_mirror: the other quad of the 8
  x = fmaxf(x, dpp_get<0x140>(x));   // row_mirror: the other half of the 16
  return x;
}
__device__ __forceinline__ float row16_sum(float x) {
  x += dpp_get<0xB1>(x);
  x += dpp_get<0x4E>(x);
  x += dpp_get<0x141>(x);
  x += dpp_get<0x140>(x);
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

// The item sizes the planning kernel chooses from when none is set: multiples of one pass of a workgroup's waves.
constexpr int kAutoParts = 7;
__host__ __device__ constexpr int32_t auto_part(int i) {
  return i == 0 ? 512 : i == 1 ? 768 : i == 2 ? 1024 : i == 3 ? 1536 : i == 4 ? 2048 : i == 5 ? 3072 : 4096;
}

// ---- planning: the list of work items ------------------------------------------------------------------
// items[i] = {sequence | part << 16, context length of the sequence}: item `part` covers the tokens
// [part * part_tokens, min((part + 1) * part_tokens, context)).  hdr[0] = number of items.  Full items
// (part_tokens tokens) come first, then one shorter item per sequence whose length is not a multiple of
// part_tokens (or is <= 0, so that its output is still written), longest first.  With minus = 1 "context" is the
// context without its last token.  hdr[1] = part_tokens: the given one, or with min_units > 0 the one chosen
// here; every kernel that follows reads it from there.  Also zeroes the ticket
// counters of all layers and, if a clock table is given, resets its rows and notes the time in the row
// after the last.
__global__ __launch_bounds__(256) void k_attn_plan(const int32_t* __restrict__ ctx, int32_t batch, int32_t part_tokens,
                                                   int32_t min_units, int32_t n_kv_heads,
                                                   int32_t max_blocks, int32_t minus, uint2* __restrict__ items,
                                                   int32_t* __restrict__ hdr, uint32_t* __restrict__ counters,
                                                   int32_t n_counters, uint32_t* __restrict__ err,
                                                   unsigned long long* __restrict__ clock) {
  __shared__ int32_t s_off[kMaxPlanBatch];   // first full item of the sequence
  __shared__ int32_t s_nf[kMaxPlanBatch];
  __shared__ int32_t s_ctx[kMaxPlanBatch];  // context length, clamped to [0, what the table can name]
  __shared__ int32_t s_rem[kMaxPlanBatch];   // size of the short item, -1 if none
  __shared__ int32_t s_total_full;
  __shared__ int32_t s_units[kAutoParts];    // items per candidate item size
  __shared__ int32_t s_part;
  if (threadIdx.x < kAutoParts) s_units[threadIdx.x] = 0;
  __syncthreads();
  int32_t my_units[kAutoParts] = {};
  for (int32_t b = threadIdx.x; b < batch; b += blockDim.x) {
    const int32_t raw = ctx[b];
    const int32_t full = clamp_ctx(raw, max_blocks);
    if (raw > full) atomicOr(err, PIE_DEVERR_BAD_HANDLE);   // the table cannot name that many blocks
    const int32_t c = full > 0 ? full - minus : full;       // minus = 1: the last token is not read from the cache
    s_ctx[b] = c > 0 ? c : 0;
    if (min_units > 0)
#pragma unroll
      for (int i = 0; i < kAutoParts; ++i) my_units[i] += c > 0 ? (c + auto_part(i) - 1) / auto_part(i) : 1;
  }
  // The item size, when it is not given: the largest candidate that still leaves more than min_units units
  // (items x kv heads) for the decode kernel's workgroups to share, the smallest candidate if none does.
  if (min_units > 0) {
#pragma unroll
    for (int i = 0; i < kAutoParts; ++i)
      if (my_units[i]) atomicAdd(&s_units[i], my_units[i]);
    __syncthreads();
    if (threadIdx.x == 0) {
      int32_t pick = auto_part(0);
      for (int i = 1; i < kAutoParts; ++i)
        if ((long long)s_units[i] * n_kv_heads > min_units) pick = auto_part(i);
      s_part = pick;
    }
  } else if (threadIdx.x == 0) {
    s_part = part_tokens;
  }
  __syncthreads();
  part_tokens = s_part;
  if (threadIdx.x == 0) hdr[1] = part_tokens;
  for (int32_t b = threadIdx.x; b < batch; b += blockDim.x) {
    const int32_t c = s_ctx[b];
    const int32_t nf = c > 0 ? c / part_tokens : 0;
    const int32_t rem = c > 0 ? c % part_tokens : 0;
    s_nf[b] = nf;
    s_rem[b] = (rem > 0 || c <= 0) ? rem : -1;
  }
  for (int32_t i = threadIdx.x; i < n_counters; i += blockDim.x) counters[i] = 0;
  if (clock) {                                   // one row per launch: min / max slots to their neutral values
    for (int32_t i = threadIdx.x; i < n_counters; i += blockDim.x) {
      clock[(size_t)i * kClockRow + kClockKernelStart] = ~0ull;
      clock[(size_t)i * kClockRow + kClockKernelEnd] = 0ull;
      clock[(size_t)i * kClockRow + kClockLayerEnd] = 0ull;
      clock[(size_t)i * kClockRow + kClockGrid] = 0ull;
    }
    if (threadIdx.x == 0) clock[(size_t)n_counters * kClockRow] = wall_clock64();   // the step begins
  }
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
      items[s_off[b] + p] = make_uint2((uint32_t)b | ((uint32_t)p << 16), (uint32_t)s_ctx[b]);
    const int32_t key = s_rem[b];
    if (key >= 0) {
      int32_t rank = 0;                                  // longest first, ties by sequence index
      for (int32_t o = 0; o < batch; ++o) {
        const int32_t k2 = s_rem[o];
        rank += (k2 > key || (k2 == key && o < b)) ? 1 : 0;
      }
      items[total_full + rank] = make_uint2((uint32_t)b | ((uint32_t)nf << 16), (uint32_t)s_ctx[b]);
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
  int32_t max_blocks, n_handles, n_gpu_blocks, n_slots;
  int32_t stage_valid[2];
};

__global__ __launch_bounds__(64) void k_attn_resolve(const ResolveArgs a) {
  const int32_t i = blockIdx.x;
  if (i >= a.hdr[0]) return;
  const uint2 rec = a.items[i];
  const int32_t b = (int32_t)(rec.x & 0xffffu), part = (int32_t)(rec.x >> 16);
  const int32_t tok1 = (int32_t)rec.y;
  const int32_t jb1 = tok1 > 0 ? (tok1 + kBlockTokens - 1) / kBlockTokens : 0;   // <= max_blocks
  const int32_t bpi = a.hdr[1] / kBlockTokens;   // blocks per item, as planned
  for (int32_t jj = threadIdx.x; jj < bpi; jj += blockDim.x) {
    const int32_t j = part * bpi + jj;
    const bool live = j < jb1;
    const int32_t h = live ? a.table[(size_t)b * a.max_blocks + j] : -1;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      if (!a.slots[r]) continue;
      a.slots[r][(size_t)i * bpi + jj] =
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
  int32_t max_blocks, n_kv_heads, group;
  int32_t n_parts;           // partitions the workspace has room for per (sequence, head); the item size is hdr[1]
  int32_t max_items;         // entries the item list has room for (batch x n_parts)
  unsigned long long* clock;    // this launch's row of the clock table, or NULL
  unsigned long long* clock_wg; // with it: a (first, last moment) pair per workgroup, or NULL (atomics on the row)
  // The newest token's key / value rows [B][Hkv][d], or NULL.  With them the items cover the context without
  // its last token (the planning kernel was told so), every partition's state goes to the workspace, and the
  // reduction kernel adds the last token from these rows: the attention then does not depend on the append
  // that writes the rows into the cache.
  const char* new_k;
  const char* new_v;
};

// LDS floats the MFMA kernel needs for `group` query heads per kv head
template <int HD>
constexpr size_t mfma_lds_floats(int group) {
  return (size_t)kWaves * 2 * kMaxGroup + (size_t)kWaves * group * (HD + 4);
}

#ifndef PIE_MFMA_WAVES_PER_EU
#define PIE_MFMA_WAVES_PER_EU 2
#endif

// VALU: the same kernel with both products on the vector ALU instead (group == 1 only, where they are
// matrix-vector products).  Lane (quad, i) then holds, of a K load, eight dims of token i - its share of that
// token's score, summed over the four quads - and of a V load four tokens of two dims, which it multiplies with
// those tokens' weights fetched from the lanes that own them; the output dims are summed over the quads when the
// unit ends.
template <typename E, int HD, bool SPLIT, bool VALU>
__global__ __launch_bounds__(kWaves * 64) __attribute__((amdgpu_waves_per_eu(PIE_MFMA_WAVES_PER_EU, 8)))
void k_attn_decode_mfma(const AttnArgs a) {
  using MM = Mfma<E>;
  constexpr int NKC = HD / 32;                    // 1 KiB loads per K tile and per V tile; QK MFMAs per block
  constexpr int NO = HD / 16;                     // output accumulators (16 dims x 16 heads each)
  constexpr int TILE_BYTES = kBlockTokens * HD * 2;
  constexpr int ROW = HD + 4;                     // padded LDS row of one head's accumulator
  static_assert(HD % 32 == 0, "unsupported head_dim");

  extern __shared__ __align__(16) float s_dyn[];
  __shared__ uint32_t s_ticket;
  float* s_m = s_dyn;                             // [kWaves][16]
  float* s_l = s_dyn + kWaves * kMaxGroup;        // [kWaves][16]
  float* s_acc = s_dyn + 2 * kWaves * kMaxGroup;  // [kWaves][G][ROW]

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 15, quad = lane >> 4;    // MFMA column (query head of the group) and 4-row group
  const int32_t G = a.group;
  const int32_t n_q_heads = a.n_kv_heads * G;
  const uint32_t n_kv = (uint32_t)a.n_kv_heads;
  const uint32_t max_units = (uint32_t)a.max_items * n_kv;        // what the item and slot lists have room for
  const size_t v_off = a.block_bytes / 2;
  const int32_t part_tokens = a.hdr[1];                           // the item size the planning kernel noted
  const int32_t bpi = part_tokens / kBlockTokens;                 // blocks per item, <= 64 * kWaves
  const int32_t my_n = (bpi + kWaves - 1 - wave) / kWaves;        // blocks of an item this wave may own

  // Units are handed out by tickets.  A workgroup's first two are static (its index, and its index plus the
  // grid size); the rest come from an atomic counter.  The ticket for the unit after next is requested
  // behind a unit's stream, so the next unit is always known one unit ahead: its record and slot list are
  // fetched at the start of the current unit, its first block is requested as soon as the current unit's
  // stream ends, and the merge of the current unit runs behind those loads.
  uint32_t unit = blockIdx.x;
  uint32_t next = gridDim.x + blockIdx.x;
  if (a.clock && threadIdx.x == 0) {
    const unsigned long long t = wall_clock64();
    if (a.clock_wg) {
      a.clock_wg[2 * blockIdx.x] = t;
      if (blockIdx.x == 0) a.clock[kClockGrid] = gridDim.x;
    } else {
      atomicMin(&a.clock[kClockKernelStart], t);
    }
  }

  // record and this wave's slot list of unit u; entries beyond the planned items are never used
  auto fetch_meta = [&](uint32_t u, uint2& r, int32_t& sl) {
    r = make_uint2(0, 0);
    sl = -1;
    if (u < max_units) {
      const uint32_t item = u / n_kv;
      r = a.items[item];
      if (lane < my_n) sl = a.slots[(size_t)item * bpi + wave + kWaves * lane];
    }
  };
  // this lane's part of the B operand of the first product: head `col` of the group, dims 32 kc + 8 quad ..
  auto load_q = [&](uint4 (&qr)[NKC], int32_t b, int32_t g) {
#pragma unroll
    for (int kc = 0; kc < NKC; ++kc) {
      qr[kc] = make_uint4(0, 0, 0, 0);
      const int head = VALU ? 0 : col;            // on the vector ALU every lane works for the one head
      if (head < G)
        qr[kc] = *reinterpret_cast<const uint4*>(a.q + (((size_t)b * n_q_heads + g * G + head) * HD + 32 * kc + 8 * quad) * 2);
    }
  };
  // Two register sets: while one block is consumed the next is already in flight.
  uint4 kA[NKC], vA[NKC], kB[NKC], vB[NKC];
  auto load_tile = [&](uint4 (&kr)[NKC], uint4 (&vr)[NKC], int32_t slots, int32_t it, int32_t g) {
    int32_t slot = __shfl(slots, it, 64);
    slot = slot < 0 ? 0 : slot;                                    // flagged blocks are masked when consumed
    const char* kp = a.kv_layer + (size_t)slot * a.block_bytes + (size_t)g * TILE_BYTES + (size_t)lane * 16;
#pragma unroll
    for (int i = 0; i < NKC; ++i) kr[i] = nt_load16(kp + (size_t)i * 1024);
#pragma unroll
    for (int i = 0; i < NKC; ++i) vr[i] = nt_load16(kp + v_off + (size_t)i * 1024);
  };
  // blocks of unit (r, u) this wave handles: j = jb0 + wave + kWaves * it, it < n_it (<= 0: nothing)
  auto wave_blocks = [&](const uint2& r) {
    const int32_t ctx_u = (int32_t)r.y, tok0_u = (int32_t)(r.x >> 16) * part_tokens;
    const int32_t tok1_u = min(ctx_u, tok0_u + part_tokens);
    const int32_t jb1_u = tok1_u > 0 ? (tok1_u + kBlockTokens - 1) / kBlockTokens : 0;
    return (jb1_u - tok0_u / kBlockTokens - wave + kWaves - 1) / kWaves;
  };

  uint2 rec, rec_next;
  int32_t my_slot, my_slot_next;
  uint4 qreg[NKC];
  fetch_meta(unit, rec, my_slot);
  fetch_meta(next, rec_next, my_slot_next);
  const uint32_t n_units = (uint32_t)a.hdr[0] * n_kv;              // <= max_units
  if (unit < n_units) {
    load_q(qreg, (int32_t)(rec.x & 0xffffu), (int32_t)(unit % n_kv));
    if (wave_blocks(rec) > 0) load_tile(kA, vA, my_slot, 0, (int32_t)(unit % n_kv));
  }

  while (unit < n_units) {                       // every workgroup ends on a ticket past the last unit
    const int32_t g = (int32_t)(unit % n_kv);
    const int32_t b = (int32_t)(rec.x & 0xffffu), part = (int32_t)(rec.x >> 16);
    const int32_t ctx_b = (int32_t)rec.y;                          // clamped context length of the sequence
    const int32_t tok0 = part * part_tokens;
    const int32_t tok1 = min(ctx_b, tok0 + part_tokens);         // <= tok0 only for an empty sequence
    const int32_t np_b = ctx_b > 0 ? (ctx_b + part_tokens - 1) / part_tokens : 1;   // partitions of the sequence
    const int32_t hq0 = g * G;
    const int32_t jb0 = tok0 / kBlockTokens;
    const int32_t n_it = wave_blocks(rec);                         // <= my_n <= 64

    float m = kNegBig, l = 0.f;                   // running max of head `col`; this lane's share of the sum
    f32x4 o[NO];
#pragma unroll
    for (int n = 0; n < NO; ++n) o[n] = f32x4{0.f, 0.f, 0.f, 0.f};
    float ov[NKC][2];                             // VALU: dims 32 i + (lane & 15) and 16 further, this quad's tokens
#pragma unroll
    for (int i = 0; i < NKC; ++i) ov[i][0] = ov[i][1] = 0.f;

    // VALU form of one block: lane (quad, i = lane & 15).  K load kc holds token i, dims 32 kc + 8 quad ..;
    // V load holds tokens 4 quad .. 4 quad + 3 of dims 32 ld + i (x, y) and 32 ld + 16 + i (z, w).
    auto consume_valu = [&](uint4 (&kr)[NKC], uint4 (&vr)[NKC], int32_t it) {
      const int32_t t_first = (jb0 + wave + kWaves * it) * kBlockTokens;
      const bool present = __shfl(my_slot, it, 64) >= 0;
      const int32_t limit = present ? tok1 : 0;
      float d = 0.f;
#pragma unroll
      for (int kc = 0; kc < NKC; ++kc) {
        d = Dot2<E>::fma2(kr[kc].x, qreg[kc].x, d);
        d = Dot2<E>::fma2(kr[kc].y, qreg[kc].y, d);
        d = Dot2<E>::fma2(kr[kc].z, qreg[kc].z, d);
        d = Dot2<E>::fma2(kr[kc].w, qreg[kc].w, d);
      }
      float sc = quad16_sum(d) * a.scale_log2e;   // score of token t_first + i, on all four lanes of the token
      if (t_first + col >= limit) sc = -INFINITY;
      if (t_first + kBlockTokens > limit) {       // garbage rows must not reach the sum
        const int32_t t_lane = t_first + 4 * quad;
        uint32_t keep_lo = 0, keep_hi = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const uint32_t bits = t_lane + r < limit ? (0xffffu << (16 * (r & 1))) : 0u;
          if (r < 2) keep_lo |= bits; else keep_hi |= bits;
        }
#pragma unroll
        for (int i = 0; i < NKC; ++i) {
          vr[i].x &= keep_lo; vr[i].y &= keep_hi; vr[i].z &= keep_lo; vr[i].w &= keep_hi;
        }
      }
      const float m_new = fmaxf(m, row16_max(sc));           // the same on every lane of the wave
      if (m_new > m) {
        const float corr = __builtin_amdgcn_exp2f(m - m_new);
        l *= corr;
#pragma unroll
        for (int i = 0; i < NKC; ++i) { ov[i][0] *= corr; ov[i][1] *= corr; }
        m = m_new;
      }
      const float p = __builtin_amdgcn_exp2f(sc - m);
      l += p;                                     // token i only; summed over the sixteen tokens when the unit ends
      f32x4 pq;                                   // the weights of this quad's four tokens
#pragma unroll
      for (int r = 0; r < 4; ++r) pq[r] = __shfl(p, 4 * quad + r, 64);
      const uint2 p_hi = MM::round(pq);
      uint2 p_lo = make_uint2(0, 0);
      if (SPLIT) {
        const f32x4 back = MM::widen(p_hi);
        f32x4 rest;
#pragma unroll
        for (int r = 0; r < 4; ++r) rest[r] = pq[r] - back[r];
        p_lo = MM::round(rest);
      }
#pragma unroll
      for (int i = 0; i < NKC; ++i) {
        ov[i][0] = Dot2<E>::fma2(vr[i].x, p_hi.x, ov[i][0]);
        ov[i][0] = Dot2<E>::fma2(vr[i].y, p_hi.y, ov[i][0]);
        ov[i][1] = Dot2<E>::fma2(vr[i].z, p_hi.x, ov[i][1]);
        ov[i][1] = Dot2<E>::fma2(vr[i].w, p_hi.y, ov[i][1]);
        if (SPLIT) {
          ov[i][0] = Dot2<E>::fma2(vr[i].x, p_lo.x, ov[i][0]);
          ov[i][0] = Dot2<E>::fma2(vr[i].y, p_lo.y, ov[i][0]);
          ov[i][1] = Dot2<E>::fma2(vr[i].z, p_lo.x, ov[i][1]);
          ov[i][1] = Dot2<E>::fma2(vr[i].w, p_lo.y, ov[i][1]);
        }
      }
    };

    auto consume = [&](uint4 (&kr)[NKC], uint4 (&vr)[NKC], int32_t it) {
      const int32_t t_first = (jb0 + wave + kWaves * it) * kBlockTokens;      // first token of the block
      const bool present = __shfl(my_slot, it, 64) >= 0;
      const int32_t limit = present ? tok1 : 0;                               // a missing block contributes nothing

      f32x4 s = {0.f, 0.f, 0.f, 0.f};             // s[r]: token t_first + 4 quad + r, head col
#pragma unroll
      for (int kc = 0; kc < NKC; ++kc) s = MM::qk(kr[kc], qreg[kc], s);
#pragma unroll
      for (int r = 0; r < 4; ++r) s[r] *= a.scale_log2e;
      if (t_first + kBlockTokens > limit) {       // the block holds rows beyond the context
        const int32_t t_lane = t_first + 4 * quad;
        uint32_t keep_lo = 0, keep_hi = 0;        // 16-bit masks of tokens (0, 1) and (2, 3) of this lane's quad
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const bool valid = t_lane + r < limit;
          s[r] = valid ? s[r] : -INFINITY;
          const uint32_t bits = valid ? (0xffffu << (16 * (r & 1))) : 0u;
          if (r < 2) keep_lo |= bits; else keep_hi |= bits;
        }
#pragma unroll
        for (int i = 0; i < NKC; ++i) {           // garbage rows must not reach the sum
          vr[i].x &= keep_lo; vr[i].y &= keep_hi; vr[i].z &= keep_lo; vr[i].w &= keep_hi;
        }
      }
      const float mx = quad16_max(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])));
      const float m_new = fmaxf(m, mx);
      if (__builtin_amdgcn_ballot_w64(m_new > m) != 0) {              // some head's maximum moved: rescale
        const float corr = __builtin_amdgcn_exp2f(m - m_new);
        l *= corr;
#pragma unroll
        for (int n = 0; n < NO; ++n)
#pragma unroll
          for (int r = 0; r < 4; ++r) o[n][r] *= corr;
        m = m_new;
      }
      f32x4 p;
#pragma unroll
      for (int r = 0; r < 4; ++r) p[r] = __builtin_amdgcn_exp2f(s[r] - m);
      l += (p[0] + p[1]) + (p[2] + p[3]);
      const uint2 p_hi = MM::round(p);
      uint2 p_lo = make_uint2(0, 0);
      if (SPLIT) {
        const f32x4 back = MM::widen(p_hi);
        f32x4 rest;
#pragma unroll
        for (int r = 0; r < 4; ++r) rest[r] = p[r] - back[r];
        p_lo = MM::round(rest);
      }
#pragma unroll
      for (int i = 0; i < NKC; ++i) {
        const uint2 v0 = make_uint2(vr[i].x, vr[i].y), v1 = make_uint2(vr[i].z, vr[i].w);
        o[2 * i] = MM::pv(v0, p_hi, o[2 * i]);
        o[2 * i + 1] = MM::pv(v1, p_hi, o[2 * i + 1]);
        if (SPLIT) {
          o[2 * i] = MM::pv(v0, p_lo, o[2 * i]);
          o[2 * i + 1] = MM::pv(v1, p_lo, o[2 * i + 1]);
        }
      }
    };

    // The ticket after next is requested half way through the stream: late enough that the counter is not
    // hit by every workgroup at once, early enough that the answer is there when the unit ends.  Block 0 of
    // the unit is already on its way in kA / vA.
    uint32_t after_next = 0;
    const int32_t it_ticket = n_it > 2 ? ((n_it / 2) & ~1) : 0;
    for (int32_t it = 0; it < n_it; it += 2) {
      if (it == it_ticket && threadIdx.x == 0) after_next = 2 * gridDim.x + atomicAdd(a.counter, 1u);
      if (it + 1 < n_it) load_tile(kB, vB, my_slot, it + 1, g);
      if constexpr (VALU) consume_valu(kA, vA, it); else consume(kA, vA, it);
      if (it + 1 < n_it) {
        if (it + 2 < n_it) load_tile(kA, vA, my_slot, it + 2, g);
        if constexpr (VALU) consume_valu(kB, vB, it + 1); else consume(kB, vB, it + 1);
      }
    }
    if (n_it <= 0 && threadIdx.x == 0) after_next = 2 * gridDim.x + atomicAdd(a.counter, 1u);

    // behind the stream: the next unit's first block and query rows arrive while this unit's result is merged
    if (next < n_units) {
      const int32_t g_next = (int32_t)(next % n_kv);
      if (wave_blocks(rec_next) > 0) load_tile(kA, vA, my_slot_next, 0, g_next);
      load_q(qreg, (int32_t)(rec_next.x & 0xffffu), g_next);
    }

    // merge the kWaves partial states: lane (quad, col) holds O[16 n + 4 quad + r][head col]
    if constexpr (VALU) {
      l = row16_sum(l);                           // over the sixteen tokens of a block position
#pragma unroll
      for (int i = 0; i < NKC; ++i) {             // over the four quads' tokens
        ov[i][0] = quad16_sum(ov[i][0]);
        ov[i][1] = quad16_sum(ov[i][1]);
      }
      if (lane == 0) {
        s_m[wave * kMaxGroup] = m;
        s_l[wave * kMaxGroup] = l;
      }
      if (quad == 0) {
        float* row = s_acc + (size_t)wave * G * ROW;
#pragma unroll
        for (int i = 0; i < NKC; ++i) {
          row[32 * i + col] = ov[i][0];
          row[32 * i + 16 + col] = ov[i][1];
        }
      }
    } else {
    l = quad16_sum(l);
    if (col < G) {
      if (quad == 0) {
        s_m[wave * kMaxGroup + col] = m;
        s_l[wave * kMaxGroup + col] = l;
      }
      float* row = s_acc + ((size_t)wave * G + col) * ROW + 4 * quad;
#pragma unroll
      for (int n = 0; n < NO; ++n) *reinterpret_cast<f32x4*>(row + 16 * n) = o[n];
    }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < G * HD; idx += kWaves * 64) {
      const int h = idx / HD, dim = idx % HD;
      float M = s_m[h];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) M = fmaxf(M, s_m[w * kMaxGroup + h]);
      float L = 0.f, A = 0.f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const float wt = __builtin_amdgcn_exp2f(s_m[w * kMaxGroup + h] - M);
        L = fmaf(wt, s_l[w * kMaxGroup + h], L);
        A = fmaf(wt, s_acc[((size_t)w * G + h) * ROW + dim], A);
      }
      const size_t orow = (size_t)b * n_q_heads + hq0 + h;
      if (np_b == 1 && !a.new_k) {               // the only partition of its sequence: this is the result
        store_elem<E>(a.out, orow * HD + dim, L > 0.f ? A / L : 0.f);
      } else {
        float* w = a.ws + (orow * a.n_parts + part) * (HD + 2);
        if (dim == 0) {
          w[0] = M;
          w[1] = L;
        }
        w[2 + dim] = A;
      }
    }
    if (threadIdx.x == 0) s_ticket = after_next;
    __syncthreads();                             // merge buffers free again; the new ticket is visible
    unit = next;
    next = s_ticket;
    rec = rec_next;
    my_slot = my_slot_next;
    __syncthreads();                             // all have read the ticket before it is overwritten
    fetch_meta(next, rec_next, my_slot_next);    // consumed when this unit's stream ends
  }
  if (a.clock && threadIdx.x == 0) {
    const unsigned long long t = wall_clock64();
    if (a.clock_wg) a.clock_wg[2 * blockIdx.x + 1] = t;
    else atomicMax(&a.clock[kClockKernelEnd], t);
  }
}

// Calibration: reads exactly the K and V tiles the decode kernel reads for the planned items, in the same
// order and with the same loads (units by ticket, wave w takes blocks w, w + kWaves, ..., two blocks in
// flight), and does nothing with them but fold them into a word nobody looks at.  Its rate is what this
// access pattern can stream at; the decode kernel is measured against it as well as against the HBM peak.
template <int NL>                                 // 1 KiB loads per tile
__global__ __launch_bounds__(kWaves * 64) void k_stream_probe(const AttnArgs a, size_t tile_bytes, uint32_t* sink) {
  __shared__ uint32_t s_ticket;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t n_kv = (uint32_t)a.n_kv_heads;
  const uint32_t n_units = (uint32_t)a.hdr[0] * n_kv;
  const size_t v_off = a.block_bytes / 2;
  const int32_t part_tokens = a.hdr[1];
  const int32_t bpi = part_tokens / kBlockTokens;
  const int32_t my_n = (bpi + kWaves - 1 - wave) / kWaves;
  u32x4 acc = {0, 0, 0, 0};
  uint32_t unit = blockIdx.x;
  while (unit < n_units) {                       // every workgroup ends on a ticket past the last unit
    const uint32_t item = unit / n_kv;
    const uint2 rec = a.items[item];
    int32_t my_slot = -1;
    if (lane < my_n) my_slot = a.slots[(size_t)item * bpi + wave + kWaves * lane];
    const int32_t ctx_u = (int32_t)rec.y, tok0 = (int32_t)(rec.x >> 16) * part_tokens;
    const int32_t tok1 = min(ctx_u, tok0 + part_tokens);
    const int32_t jb1 = tok1 > 0 ? (tok1 + kBlockTokens - 1) / kBlockTokens : 0;
    const int32_t n_it = (jb1 - tok0 / kBlockTokens - wave + kWaves - 1) / kWaves;
    const size_t head_off = (size_t)(unit % n_kv) * tile_bytes + (size_t)lane * 16;
    u32x4 ta[2 * NL], tb[2 * NL];
    auto load = [&](u32x4 (&t)[2 * NL], int32_t it) {
      int32_t slot = __shfl(my_slot, it, 64);
      slot = slot < 0 ? 0 : slot;
      const char* kp = a.kv_layer + (size_t)slot * a.block_bytes + head_off;
#pragma unroll
      for (int i = 0; i < NL; ++i) t[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kp + (size_t)i * 1024));
#pragma unroll
      for (int i = 0; i < NL; ++i)
        t[NL + i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kp + v_off + (size_t)i * 1024));
    };
    auto fold = [&](u32x4 (&t)[2 * NL]) {
#pragma unroll
      for (int i = 0; i < 2 * NL; ++i) acc ^= t[i];
    };
    if (n_it > 0) load(ta, 0);
    for (int32_t it = 0; it < n_it; it += 2) {
      if (it + 1 < n_it) load(tb, it + 1);
      fold(ta);
      if (it + 1 < n_it) {
        if (it + 2 < n_it) load(ta, it + 2);
        fold(tb);
      }
    }
    if (threadIdx.x == 0) s_ticket = gridDim.x + atomicAdd(a.counter, 1u);
    __syncthreads();
    unit = s_ticket;
    __syncthreads();
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) *sink = 1;   // keeps the loads alive
}

// fp32 caches.  One workgroup per (item, query head); wave w takes blocks w, w + kWaves, ...  Lane
// (quad, row) = (lane / 16, lane % 16): for K it holds token `row` of the block and the 4-dim vectors
// 4 i + quad; for V it holds dim 16 n + row and the tokens 4 quad .. 4 quad + 3.
template <int HD>
__global__ __launch_bounds__(kWaves * 64) void k_attn_decode_f32(const AttnArgs a) {
  constexpr int NLD = HD / 16;                    // 1 KiB loads per K tile and per V tile
  constexpr int TILE_BYTES = kBlockTokens * HD * 4;
  __shared__ float s_m[kWaves], s_l[kWaves];
  __shared__ float s_acc[kWaves][HD];

  const int32_t item = blockIdx.x;
  if (item >= a.hdr[0]) return;                   // uniform over the workgroup
  if (a.clock && threadIdx.x == 0) atomicMin(&a.clock[kClockKernelStart], wall_clock64());
  const int32_t hq = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = lane & 15, quad = lane >> 4;
  const int32_t G = a.group;
  const int32_t n_q_heads = a.n_kv_heads * G;
  const int32_t g = hq / G;
  const int32_t part_tokens = a.hdr[1];
  const int32_t bpi = part_tokens / kBlockTokens;
  const int32_t my_n = (bpi + kWaves - 1 - wave) / kWaves;
  const uint2 rec = a.items[item];
  const int32_t b = (int32_t)(rec.x & 0xffffu), part = (int32_t)(rec.x >> 16);
  const int32_t ctx_b = (int32_t)rec.y;           // clamped context length of the sequence
  const int32_t tok0 = part * part_tokens, tok1 = min(ctx_b, tok0 + part_tokens);
  const int32_t np_b = ctx_b > 0 ? (ctx_b + part_tokens - 1) / part_tokens : 1;
  const int32_t jb0 = tok0 / kBlockTokens;
  const int32_t jb1 = tok1 > 0 ? (tok1 + kBlockTokens - 1) / kBlockTokens : 0;
  const int32_t n_it = (jb1 - jb0 - wave + kWaves - 1) / kWaves;
  int32_t my_slot = -1;
  if (lane < my_n) my_slot = a.slots[(size_t)item * bpi + wave + kWaves * lane];

  float qf[NLD][4];
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    const float4 t = *reinterpret_cast<const float4*>(a.q + (((size_t)b * n_q_heads + hq) * HD + 4 * (4 * i + quad)) * 4);
    qf[i][0] = t.x * a.scale_log2e; qf[i][1] = t.y * a.scale_log2e;
    qf[i][2] = t.z * a.scale_log2e; qf[i][3] = t.w * a.scale_log2e;
  }
  float m = kNegBig, l = 0.f, acc[NLD];
#pragma unroll
  for (int n = 0; n < NLD; ++n) acc[n] = 0.f;
  const size_t v_off = a.block_bytes / 2;
  const size_t head_off = (size_t)g * TILE_BYTES + (size_t)lane * 16;

  for (int32_t it = 0; it < n_it; ++it) {
    int32_t slot = __shfl(my_slot, it, 64);
    const bool present = slot >= 0;
    slot = present ? slot : 0;
    const int32_t limit = present ? tok1 : 0;
    const int32_t t_first = (jb0 + wave + kWaves * it) * kBlockTokens;
    const char* kp = a.kv_layer + (size_t)slot * a.block_bytes + head_off;
    float d = 0.f;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const uint4 r = nt_load16(kp + (size_t)i * 1024);
      d = fmaf(qf[i][0], __uint_as_float(r.x), d);
      d = fmaf(qf[i][1], __uint_as_float(r.y), d);
      d = fmaf(qf[i][2], __uint_as_float(r.z), d);
      d = fmaf(qf[i][3], __uint_as_float(r.w), d);
    }
    float s = quad16_sum(d);                      // score of token t_first + row, on all four lanes of the token
    if (t_first + row >= limit) s = -INFINITY;
    const float m_new = fmaxf(m, row16_max(s));
    const float corr = __builtin_amdgcn_exp2f(m - m_new);
    const float p = __builtin_amdgcn_exp2f(s - m_new);
    l = l * corr + p;                             // this lane's token only; summed over the row at the end
    m = m_new;
    float pt[4];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) pt[tt] = __shfl(p, 4 * quad + tt, 64);
#pragma unroll
    for (int n = 0; n < NLD; ++n) {
      const uint4 r = nt_load16(kp + v_off + (size_t)n * 1024);
      const uint32_t w[4] = {r.x, r.y, r.z, r.w};
      float x = acc[n] * corr;
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        const bool valid = t_first + 4 * quad + tt < limit;        // garbage rows must not reach the sum
        x = fmaf(pt[tt], valid ? __uint_as_float(w[tt]) : 0.f, x);
      }
      acc[n] = x;
    }
  }
  l = row16_sum(l);
#pragma unroll
  for (int n = 0; n < NLD; ++n) acc[n] = quad16_sum(acc[n]);
  if (lane == 0) {
    s_m[wave] = m;
    s_l[wave] = l;
  }
  if (quad == 0) {
#pragma unroll
    for (int n = 0; n < NLD; ++n) s_acc[wave][16 * n + row] = acc[n];
  }
  __syncthreads();
  for (int dim = threadIdx.x; dim < HD; dim += kWaves * 64) {
    float M = s_m[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) M = fmaxf(M, s_m[w]);
    float L = 0.f, A = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float wt = __builtin_amdgcn_exp2f(s_m[w] - M);
      L = fmaf(wt, s_l[w], L);
      A = fmaf(wt, s_acc[w][dim], A);
    }
    const size_t orow = (size_t)b * n_q_heads + hq;
    if (np_b == 1 && !a.new_k) {                 // the only partition of its sequence: this is the result
      store_elem<F32>(a.out, orow * HD + dim, L > 0.f ? A / L : 0.f);
    } else {
      float* w = a.ws + (orow * a.n_parts + part) * (HD + 2);
      if (dim == 0) {
        w[0] = M;
        w[1] = L;
      }
      w[2 + dim] = A;
    }
  }
  if (a.clock && threadIdx.x == 0) atomicMax(&a.clock[kClockKernelEnd], wall_clock64());
}

// Reduction over the partitions of one (sequence, query head): out = sum_s 2^(m_s - M) acc_s / sum_s 2^(m_s - M) l_s.
// With the newest token's rows given, that token is one more partition, (q . k_new, 1, v_new), computed here:
// s = q . k_new in the log2 domain like the partitions' maxima; the rows are requested first and used after the
// partitions have been merged.
//
// Two forms.  k_attn_reduce_heads, for up to eight partitions per sequence: head_dim / 2 threads per query head,
// two dims each, 512 / head_dim heads per workgroup, no LDS and no barrier (the launch is as short as its number
// of workgroups allows: the 8B workload has 8 192 rows).  k_attn_reduce, for long contexts: 256 threads per
// head, thread (sub, dim) = (tid / HD, tid % HD) merging the partitions sub, sub + 256/HD, ... online, four
// loads in flight, and the 256/HD partial merges meet in LDS.

struct ReduceRow {
  int32_t np;        // partitions to merge
  bool add_new;      // and the newest token
  bool skip;         // nothing to do: a lone partition wrote the result itself
};
__device__ __forceinline__ ReduceRow reduce_row(const AttnArgs& a, int32_t b) {
  const int32_t full = clamp_ctx(a.ctx[b], a.max_blocks);
  const bool with_new = a.new_k != nullptr;
  const int32_t ctx = with_new && full > 0 ? full - 1 : full;   // the tokens the partitions covered
  const int32_t part_tokens = a.hdr[1];
  int32_t np = ctx <= 0 ? 1 : (ctx + part_tokens - 1) / part_tokens;
  if (np > a.n_parts) np = a.n_parts;
  return {np, with_new && full > 0, np <= 1 && !with_new};
}

template <typename E, int HD>
__global__ __launch_bounds__(256) void k_attn_reduce_heads(const AttnArgs a, int32_t n_q_heads) {
  constexpr int TPH = HD / 2;                     // threads per head: a wave or half a wave
  constexpr int HPW = 256 / TPH;
  constexpr int UNR = 4;
  static_assert(TPH == 64 || TPH == 32, "a head's threads must be a wave or half a wave");
  const int32_t b = blockIdx.y;
  const int d0 = 2 * (threadIdx.x % TPH);
  const int32_t hq = (int32_t)blockIdx.x * HPW + threadIdx.x / TPH;
  const ReduceRow r = reduce_row(a, b);
  if (r.skip) return;
  if (hq < n_q_heads) {
    const size_t row = (size_t)b * n_q_heads + hq;
    float qk = 0.f;
    float2 v_new = make_float2(0.f, 0.f);
    if (r.add_new) {
      const size_t kv_row = ((size_t)b * a.n_kv_heads + hq / a.group) * HD;
      const float2 q2 = load_elem2<E>(a.q, row * HD + d0), k2 = load_elem2<E>(a.new_k, kv_row + d0);
      qk = fmaf(q2.x, k2.x, q2.y * k2.y);
      v_new = load_elem2<E>(a.new_v, kv_row + d0);
    }
    const float* w = a.ws + row * a.n_parts * (HD + 2);
    float M = kNegBig, L = 0.f;
    float2 A = make_float2(0.f, 0.f);
    for (int32_t s0 = 0; s0 < r.np; s0 += UNR) {
      float mi[UNR], li[UNR];
      float2 ai[UNR];
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const bool live = s0 + u < r.np;
        const float* wp = w + (size_t)(live ? s0 + u : s0) * (HD + 2);
        mi[u] = live ? wp[0] : kNegBig;
        li[u] = live ? wp[1] : 0.f;
        ai[u] = live ? *reinterpret_cast<const float2*>(wp + 2 + d0) : make_float2(0.f, 0.f);
      }
      float m_new = M;
#pragma unroll
      for (int u = 0; u < UNR; ++u) m_new = fmaxf(m_new, mi[u]);
      const float corr = __builtin_amdgcn_exp2f(M - m_new);
      L *= corr;
      A.x *= corr;
      A.y *= corr;
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const float wt = __builtin_amdgcn_exp2f(mi[u] - m_new);
        L = fmaf(wt, li[u], L);
        A.x = fmaf(wt, ai[u].x, A.x);
        A.y = fmaf(wt, ai[u].y, A.y);
      }
      M = m_new;
    }
    if (r.add_new) {
      float d = row16_sum(qk);                    // over the head's threads: rows of 16 lanes, then the rows
      if constexpr (TPH == 64) d = quad16_sum(d);
      else d += __shfl_xor(d, 16, 64);
      const float s_new = d * a.scale_log2e;
      const float m2 = fmaxf(M, s_new);
      const float w_old = __builtin_amdgcn_exp2f(M - m2), w_new = __builtin_amdgcn_exp2f(s_new - m2);
      L = fmaf(L, w_old, w_new);
      A.x = fmaf(A.x, w_old, w_new * v_new.x);
      A.y = fmaf(A.y, w_old, w_new * v_new.y);
    }
    const float inv = L > 0.f ? 1.f / L : 0.f;
    store_elem2<E>(a.out, row * HD + d0, make_float2(L > 0.f ? A.x * inv : 0.f, L > 0.f ? A.y * inv : 0.f));
  }
  // the last workgroups dispatched are the last to end, to within a few of them: those of the last sequence
  // and one per 16 sequences note the time
  if (a.clock && threadIdx.x == 0 && (b == (int32_t)gridDim.y - 1 || (blockIdx.x == 0 && (b & 15) == 15)))
    atomicMax(&a.clock[kClockLayerEnd], wall_clock64());
}

template <typename E, int HD>
__global__ __launch_bounds__(256) void k_attn_reduce(const AttnArgs a, int32_t n_q_heads) {
  constexpr int NSUB = 256 / HD;
  constexpr int UNR = 4;
  constexpr int WPH = (HD + 63) / 64;             // waves that hold a head's q . k_new products
  __shared__ float s_M[NSUB], s_L[NSUB], s_A[NSUB][HD];
  __shared__ float s_dot[WPH];
  const int32_t hq = blockIdx.x, b = blockIdx.y;
  const int dim = threadIdx.x % HD, sub = threadIdx.x / HD;
  const ReduceRow r = reduce_row(a, b);
  if (r.skip) return;
  const size_t row = (size_t)b * n_q_heads + hq;
  float qk = 0.f, v_new = 0.f;
  if (r.add_new && sub == 0) {
    const size_t kv_row = ((size_t)b * a.n_kv_heads + hq / a.group) * HD;
    qk = load_elem<E>(a.q, row * HD + dim) * load_elem<E>(a.new_k, kv_row + dim);
    v_new = load_elem<E>(a.new_v, kv_row + dim);
  }
  const float* w = a.ws + row * a.n_parts * (HD + 2);
  float M = kNegBig, L = 0.f, A = 0.f;
  for (int32_t s0 = sub; s0 < r.np; s0 += NSUB * UNR) {
    float mi[UNR], li[UNR], ai[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int32_t sp = s0 + u * NSUB;
      const bool live = sp < r.np;
      const float* wp = w + (size_t)(live ? sp : s0) * (HD + 2);
      mi[u] = live ? wp[0] : kNegBig;
      li[u] = live ? wp[1] : 0.f;
      ai[u] = live ? wp[2 + dim] : 0.f;
    }
    float m_new = M;
#pragma unroll
    for (int u = 0; u < UNR; ++u) m_new = fmaxf(m_new, mi[u]);
    const float corr = __builtin_amdgcn_exp2f(M - m_new);
    L *= corr;
    A *= corr;
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const float wt = __builtin_amdgcn_exp2f(mi[u] - m_new);
      L = fmaf(wt, li[u], L);
      A = fmaf(wt, ai[u], A);
    }
    M = m_new;
  }
  if (dim == 0) {
    s_M[sub] = M;
    s_L[sub] = L;
  }
  s_A[sub][dim] = A;
  if (r.add_new && sub == 0) {                   // HD / 64 waves hold the products: each leaves its sum
    const float wave_sum = quad16_sum(row16_sum(qk));
    if ((threadIdx.x & 63) == 0) s_dot[threadIdx.x >> 6] = wave_sum;
  }
  __syncthreads();
  if (sub == 0) {
    float Mt = s_M[0];
#pragma unroll
    for (int i = 1; i < NSUB; ++i) Mt = fmaxf(Mt, s_M[i]);
    float Lt = 0.f, At = 0.f;
#pragma unroll
    for (int i = 0; i < NSUB; ++i) {
      const float wt = __builtin_amdgcn_exp2f(s_M[i] - Mt);
      Lt = fmaf(wt, s_L[i], Lt);
      At = fmaf(wt, s_A[i][dim], At);
    }
    if (r.add_new) {
      float d = s_dot[0];
#pragma unroll
      for (int i = 1; i < WPH; ++i) d += s_dot[i];
      const float s_new = d * a.scale_log2e;
      const float m2 = fmaxf(Mt, s_new);
      const float w_old = __builtin_amdgcn_exp2f(Mt - m2), w_new = __builtin_amdgcn_exp2f(s_new - m2);
      Lt = fmaf(Lt, w_old, w_new);
      At = fmaf(At, w_old, w_new * v_new);
    }
    store_elem<E>(a.out, row * HD + dim, Lt > 0.f ? At / Lt : 0.f);
  }
  if (a.clock && threadIdx.x == 0 && (b == (int32_t)gridDim.y - 1 || (hq == 0 && (b & 15) == 15)))
    atomicMax(&a.clock[kClockLayerEnd], wall_clock64());
}

// ---- dispatch ----------------------------------------------------------------------------------------

bool attn_config_supported(const pie_config& c) {
  if (c.block_tokens != kBlockTokens || c.dtype < 0 || c.dtype > 2) return false;
  if (c.head_dim != 64 && c.head_dim != 128) return false;
  const int32_t g = c.n_q_heads / c.n_kv_heads;
  if (c.dtype != PIE_DTYPE_F32 && g > kMaxGroup) return false;
  return c.max_batch <= kMaxPlanBatch && c.max_blocks_per_seq <= (1 << 19);
}

static size_t max_parts_for(int32_t max_blocks) {
  const size_t mp = ((size_t)max_blocks * kBlockTokens + kMinPartTokens - 1) / kMinPartTokens;
  return mp ? mp : 1;
}
static size_t max_parts_of(const pie_config& c) { return max_parts_for(c.max_blocks_per_seq); }

size_t attn_workspace_floats(const pie_config& c) {
  return (size_t)c.max_batch * c.n_q_heads * max_parts_of(c) * (c.head_dim + 2);
}

// Blocks of slot lists one region needs: every item lists part_tokens / 16 slots, and a sequence's items
// cover its blocks rounded up to a whole item.
static size_t slot_list_ints(int32_t batch, int32_t max_blocks) {
  return (size_t)batch * ((size_t)max_blocks + kWaves * 64);
}

// int32 words of planning state: header, ticket counters (one per layer of a step), item records (2 words
// each), and the per-item slot lists of the two staging regions
static size_t plan_counter_ints(int32_t n_counters) {
  return (size_t)n_counters + ((size_t)n_counters & 1);    // keeps the item records 8-byte aligned
}

static size_t plan_ints_for(int32_t n_counters, int32_t batch, int32_t max_blocks) {
  return kPlanHdrInts + plan_counter_ints(n_counters) + 2 * (size_t)batch * max_parts_for(max_blocks) +
         2 * slot_list_ints(batch, max_blocks);
}

size_t attn_plan_ints(const pie_config& c) { return plan_ints_for(c.n_layers, c.max_batch, c.max_blocks_per_seq); }

// The pool's own scratch: the planning state and the partials carved from the caller's device buffer, laid out
// for the pool's largest batch and table width.
static AttnWork pool_work(const pie_pool* p) {
  AttnWork w;
  w.plan = p->d_plan;
  w.ws = p->d_ws;
  w.ws_floats = p->ws_floats;
  w.n_counters = p->cfg.n_layers;
  w.lay_batch = p->cfg.max_batch;
  w.lay_max_blocks = p->cfg.max_blocks_per_seq;
  return w;
}

static int32_t* plan_hdr(const AttnWork& w) { return w.plan; }
static uint32_t* plan_counters(const AttnWork& w) { return reinterpret_cast<uint32_t*>(w.plan + kPlanHdrInts); }
static size_t plan_items_off(const AttnWork& w) { return kPlanHdrInts + plan_counter_ints(w.n_counters); }
static uint2* plan_items(const AttnWork& w) { return reinterpret_cast<uint2*>(w.plan + plan_items_off(w)); }
static int32_t* plan_slots(const AttnWork& w, int region) {
  return w.plan + plan_items_off(w) + 2 * (size_t)w.lay_batch * max_parts_for(w.lay_max_blocks) +
         (size_t)region * slot_list_ints(w.lay_batch, w.lay_max_blocks);
}

// Item size: a multiple of one pass of the workgroup's waves, at most 64 blocks per wave.  With no size set
// (attn_partition 0) the planning kernel chooses one of auto_part(); the host then sizes grids and the
// workspace for the smallest of them, which has the most items.
static int32_t part_tokens_of(const pie_pool* p) {
  int32_t part = p->attn_partition;
  if (part <= 0) return auto_part(0);
  const int32_t quantum = kWaves * kBlockTokens;
  if (part < kMinPartTokens) part = kMinPartTokens;
  part = (part + quantum - 1) / quantum * quantum;
  if (part > quantum * 64) part = quantum * 64;
  return part;
}

int launch_attn_plan(const pie_pool* p, const int32_t* d_ctx, int32_t batch, int32_t max_blocks, hipStream_t s,
                     bool reset_clock, const AttnWork* work, bool without_last) {
  const AttnWork w = work ? *work : pool_work(p);
  if (batch > kMaxPlanBatch || batch > w.lay_batch || max_blocks > w.lay_max_blocks) return PIE_EINVAL;
  // automatic item size: keep more than about eight and a half units per workgroup of the persistent decode grid
  const int32_t min_units = p->attn_partition <= 0 ? p->n_cu * 17 : 0;
  hipLaunchKernelGGL(k_attn_plan, dim3(1), dim3(256), 0, s, d_ctx, batch, part_tokens_of(p), min_units,
                     p->cfg.n_kv_heads, max_blocks, without_last ? 1 : 0, plan_items(w),
                     plan_hdr(w), plan_counters(w), w.n_counters, p->d_err, reset_clock ? p->d_clock : nullptr);
  PIE_HIP(hipGetLastError());
  return PIE_OK;
}

int launch_attn_resolve(const pie_pool* p, const int32_t* d_table, const int32_t* d_ctx, int32_t batch,
                        int32_t max_blocks, bool region0, bool valid0, bool region1, bool valid1, hipStream_t s,
                        const LayerView* view, const AttnWork* work) {
  (void)d_ctx;
  const AttnWork w = work ? *work : pool_work(p);
  if (batch > w.lay_batch || max_blocks > w.lay_max_blocks || max_blocks <= 0) return PIE_EINVAL;
  const int32_t part = part_tokens_of(p);
  ResolveArgs a;
  a.table = d_table;
  a.items = plan_items(w);
  a.hdr = plan_hdr(w);
  a.map[0] = p->d_map[0];
  a.map[1] = p->d_map[1];
  a.slots[0] = region0 ? plan_slots(w, 0) : nullptr;
  a.slots[1] = region1 ? plan_slots(w, 1) : nullptr;
  a.err = p->d_err;
  a.max_blocks = max_blocks;
  a.n_handles = p->n_handles;
  a.n_gpu_blocks = p->cfg.n_gpu_blocks;
  a.n_slots = p->cfg.n_gpu_blocks + 2 * p->cfg.n_stage_blocks;
  a.stage_valid[0] = valid0 ? 1 : 0;
  a.stage_valid[1] = valid1 ? 1 : 0;
  if (view) {                                    // one layer's own handle -> slot map, into the slot list of region 0
    if (!region0 || region1) return PIE_EINVAL;
    a.map[0] = view->map;
    a.n_handles = view->n_handles;
    a.n_gpu_blocks = a.n_slots = view->n_slots;
  }
  // one workgroup per possible item; those past the planned count return at once
  const int32_t max_items = batch * ((max_blocks * kBlockTokens + part - 1) / part);
  hipLaunchKernelGGL(k_attn_resolve, dim3(max_items), dim3(64), 0, s, a);
  PIE_HIP(hipGetLastError());
  return PIE_OK;
}

// done: an event that is to complete with this kernel (it rides on the kernel's own completion signal), or NULL
template <typename E, int HD>
static void launch_reduce(const AttnArgs& a, int32_t batch, int32_t n_q_heads, hipStream_t s, hipEvent_t done) {
  if (a.n_parts <= 8) {                           // few partitions per sequence: several heads per workgroup
    constexpr int HPW = 512 / HD;
    hipExtLaunchKernelGGL((k_attn_reduce_heads<E, HD>), dim3((n_q_heads + HPW - 1) / HPW, batch), dim3(256), 0, s,
                          nullptr, done, 0, a, n_q_heads);
  } else {
    hipExtLaunchKernelGGL((k_attn_reduce<E, HD>), dim3(n_q_heads, batch), dim3(256), 0, s, nullptr, done, 0, a,
                          n_q_heads);
  }
}

template <typename E, int HD, bool SPLIT, bool VALU = false>
static int launch_mfma(const pie_pool* p, AttnArgs a, int32_t layer_row, int32_t batch, int32_t n_q_heads,
                       hipStream_t s, hipEvent_t e0, hipEvent_t e1, hipEvent_t done) {
  const size_t lds = mfma_lds_floats<HD>(a.group) * sizeof(float);
  // as many workgroups as fit on the GPU at once; the ticket counter hands out the work
  static int wgs_per_cu[kMaxGroup + 1] = {};
  if (wgs_per_cu[a.group] == 0) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_attn_decode_mfma<E, HD, SPLIT, VALU>, kWaves * 64, lds) != hipSuccess ||
        n < 1) {
      (void)hipGetLastError();
      n = 2;
    }
    wgs_per_cu[a.group] = n;
  }
  const int grid = p->n_cu * wgs_per_cu[a.group];
  if (a.clock && grid <= kClockWgs)
    a.clock_wg = p->d_clock + ((size_t)p->cfg.n_layers + 1) * kClockRow + (size_t)layer_row * kClockWgs * 2;
  if (e0) PIE_HIP(hipEventRecord(e0, s));
  // `done` (an event that completes with the layer's last kernel) rides on that kernel's own completion
  // signal instead of a packet of its own behind it
  const bool reduce = a.n_parts > 1 || a.new_k;
  if (done && !reduce)
    hipExtLaunchKernelGGL((k_attn_decode_mfma<E, HD, SPLIT, VALU>), dim3(grid), dim3(kWaves * 64), (uint32_t)lds, s,
                          nullptr, done, 0, a);
  else
    hipLaunchKernelGGL((k_attn_decode_mfma<E, HD, SPLIT, VALU>), dim3(grid), dim3(kWaves * 64), lds, s, a);
  PIE_HIP(hipGetLastError());
  if (e1) PIE_HIP(hipEventRecord(e1, s));
  if (reduce) launch_reduce<E, HD>(a, batch, n_q_heads, s, done);
  PIE_HIP(hipGetLastError());
  return PIE_OK;
}

template <int HD>
static int launch_f32(const AttnArgs& a, int32_t batch, int32_t n_q_heads, int32_t max_items, hipStream_t s,
                      hipEvent_t e0, hipEvent_t e1, hipEvent_t done) {
  if (e0) PIE_HIP(hipEventRecord(e0, s));
  // one workgroup per possible item and query head; those past the planned count return at once
  hipLaunchKernelGGL((k_attn_decode_f32<HD>), dim3(max_items, n_q_heads), dim3(kWaves * 64), 0, s, a);
  PIE_HIP(hipGetLastError());
  if (e1) PIE_HIP(hipEventRecord(e1, s));
  if (a.n_parts > 1 || a.new_k) {
    launch_reduce<F32, HD>(a, batch, n_q_heads, s, nullptr);
    PIE_HIP(hipGetLastError());
  }
  if (done) PIE_HIP(hipEventRecord(done, s));     // the fp32 path is not tuned: an ordinary record
  return PIE_OK;
}

// Needs launch_attn_plan and launch_attn_resolve (for region layer & 1) earlier on the same stream, with the
// same batch, table width and context lengths.  d_k_new / d_v_new: the newest token's rows of this layer, taken
// from there instead of from the cache (the planning launch must have been told: without_last); NULL = the cache
// holds every token.
int launch_attn_decode(const pie_pool* p, int32_t layer, const void* d_q, int32_t max_blocks, const int32_t* d_ctx,
                       int32_t batch, void* d_out, hipStream_t s, hipEvent_t k_start, hipEvent_t k_end,
                       int32_t ticket_index, unsigned long long* clock_row, const LayerView* view, hipEvent_t done,
                       const AttnWork* work, const void* d_k_new, const void* d_v_new) {
  const pie_config& c = p->cfg;
  const AttnWork w = work ? *work : pool_work(p);
  if (((uintptr_t)d_q | (uintptr_t)d_out) % 16) return PIE_EINVAL;
  if (max_blocks <= 0) return PIE_EINVAL;
  if (c.n_gpu_blocks + 2 * c.n_stage_blocks <= 0) return PIE_EINVAL;
  const int32_t g = c.n_q_heads / c.n_kv_heads;
  const int32_t part = part_tokens_of(p);
  const int32_t max_tokens = max_blocks * kBlockTokens;
  const int32_t n_parts = (max_tokens + part - 1) / part;
  if ((size_t)batch * c.n_q_heads * n_parts * (c.head_dim + 2) > w.ws_floats) return PIE_ENOMEM;
  if (batch > w.lay_batch || max_blocks > w.lay_max_blocks) return PIE_EINVAL;

  AttnArgs a;
  a.kv_layer = view ? view->kv_base : p->d_kv + (size_t)layer * p->d_layer_stride;
  a.slots = plan_slots(w, view ? 0 : (layer & 1));
  a.items = plan_items(w);
  a.hdr = plan_hdr(w);
  // one ticket counter per launch since the last planning kernel (by default the layer's)
  if (ticket_index < 0) ticket_index = layer;
  if (ticket_index >= w.n_counters) return PIE_EINVAL;
  a.counter = plan_counters(w) + ticket_index;
  a.q = (const char*)d_q;
  a.out = (char*)d_out;
  a.ws = w.ws;
  a.ctx = d_ctx;
  a.block_bytes = p->block_bytes;
  a.scale_log2e = p->scale_log2e;
  a.max_blocks = max_blocks;
  a.n_kv_heads = c.n_kv_heads;
  a.group = g;
  a.n_parts = n_parts;
  a.max_items = batch * n_parts;
  a.clock = clock_row;
  a.clock_wg = nullptr;         // set by the launcher of a persistent grid that fits the per-workgroup words
  if ((d_k_new == nullptr) != (d_v_new == nullptr)) return PIE_EINVAL;
  if (((uintptr_t)d_k_new | (uintptr_t)d_v_new) % 8) return PIE_EINVAL;   // the reduction loads two elements at once
  a.new_k = (const char*)d_k_new;
  a.new_v = (const char*)d_v_new;
  const bool hd128 = c.head_dim == 128;
  const int32_t row = clock_row ? (int32_t)((clock_row - p->d_clock) / kClockRow) : 0;
  switch (c.dtype) {
    case PIE_DTYPE_F32: {
      return hd128 ? launch_f32<128>(a, batch, c.n_q_heads, a.max_items, s, k_start, k_end, done)
                   : launch_f32<64>(a, batch, c.n_q_heads, a.max_items, s, k_start, k_end, done);
    }
    case PIE_DTYPE_F16:
      if (g == 1 && p->attn_valu)
        return hd128 ? launch_mfma<F16, 128, false, true>(p, a, row, batch, c.n_q_heads, s, k_start, k_end, done)
                     : launch_mfma<F16, 64, false, true>(p, a, row, batch, c.n_q_heads, s, k_start, k_end, done);
      return hd128 ? launch_mfma<F16, 128, false>(p, a, row, batch, c.n_q_heads, s, k_start, k_end, done)
                   : launch_mfma<F16, 64, false>(p, a, row, batch, c.n_q_heads, s, k_start, k_end, done);
    case PIE_DTYPE_BF16:
      if (g == 1 && p->attn_valu)
        return hd128 ? launch_mfma<BF16, 128, true, true>(p, a, row, batch, c.n_q_heads, s, k_start, k_end, done)
                     : launch_mfma<BF16, 64, true, true>(p, a, row, batch, c.n_q_heads, s, k_start, k_end, done);
      return hd128 ? launch_mfma<BF16, 128, true>(p, a, row, batch, c.n_q_heads, s, k_start, k_end, done)
                   : launch_mfma<BF16, 64, true>(p, a, row, batch, c.n_q_heads, s, k_start, k_end, done);
    default: return PIE_EINVAL;
  }
}

// The calibration kernel over the same planning state (launch_attn_plan and launch_attn_resolve first).
int launch_stream_probe(const pie_pool* p, int32_t layer, int32_t max_blocks, int32_t batch, hipStream_t s) {
  const pie_config& c = p->cfg;
  if (max_blocks <= 0 || layer < 0 || layer >= c.n_layers) return PIE_EINVAL;
  const int32_t part = part_tokens_of(p);
  const AttnWork w = pool_work(p);
  AttnArgs a = {};
  a.kv_layer = p->d_kv + (size_t)layer * p->d_layer_stride;
  a.slots = plan_slots(w, layer & 1);
  a.items = plan_items(w);
  a.hdr = plan_hdr(w);
  a.counter = plan_counters(w) + layer;
  a.block_bytes = p->block_bytes;
  a.n_kv_heads = c.n_kv_heads;
  const size_t tile_bytes = (size_t)kBlockTokens * c.head_dim * p->elem_bytes;
  uint32_t* sink = p->d_err + 1;                  // a spare word of the error page
  const int grid = p->n_cu * 2;
  switch (tile_bytes / 1024) {
    case 2: hipLaunchKernelGGL((k_stream_probe<2>), dim3(grid), dim3(kWaves * 64), 0, s, a, tile_bytes, sink); break;
    case 4: hipLaunchKernelGGL((k_stream_probe<4>), dim3(grid), dim3(kWaves * 64), 0, s, a, tile_bytes, sink); break;
    case 8: hipLaunchKernelGGL((k_stream_probe<8>), dim3(grid), dim3(kWaves * 64), 0, s, a, tile_bytes, sink); break;
    default: return PIE_EINVAL;
  }
  PIE_HIP(hipGetLastError());
  return PIE_OK;
}

// ---- attention without a workspace from the caller ---------------------------------------------------
// For callers that cannot give or allocate scratch memory (code under graph capture, tight serving loops,
// harnesses that forbid allocation): the planning state and the split-context partials of one attention call
// live in a file-scope device array.  Every device the library runs on holds its own copy of the array for the
// life of the process; its address on a device is looked up once, with that device current, and only that
// address is ever handed to kernels (the array's name in host code is a host-side stand-in).

constexpr size_t kStaticScratchBytes = (size_t)40 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxScratchDevices = 64;
static char* g_scratch_ptr[kMaxScratchDevices] = {};
static std::mutex g_scratch_mutex;

// Device address of the current device's copy of the array.
int attn_static_scratch(char** out) {
  int dev = -1;
  PIE_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxScratchDevices) return PIE_EINVAL;
  std::lock_guard<std::mutex> guard(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    PIE_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return PIE_EHIP;
    g_scratch_ptr[dev] = static_cast<char*>(ptr);
  }
  *out = g_scratch_ptr[dev];
  return PIE_OK;
}

// The scratch of one call over `batch` sequences of up to `max_blocks` blocks, placed in the array: planning
// state first, partials behind it.  PIE_ENOMEM if the call needs more than the array holds.
int attn_static_work(const pie_pool* p, int32_t batch, int32_t max_blocks, AttnWork* out) {
  if (batch < 0 || batch > kMaxPlanBatch || max_blocks < 0 || max_blocks > (1 << 19)) return PIE_EINVAL;
  char* base = nullptr;
  const int rc = attn_static_scratch(&base);
  if (rc) return rc;
  const int32_t part = part_tokens_of(p);
  const size_t n_parts = ((size_t)max_blocks * kBlockTokens + part - 1) / part;
  const size_t plan_bytes = (plan_ints_for(2, batch, max_blocks) * 4 + kAlign - 1) / kAlign * kAlign;
  const size_t ws_floats = (size_t)batch * p->cfg.n_q_heads * n_parts * (p->cfg.head_dim + 2);
  if (plan_bytes > kStaticScratchBytes || ws_floats * 4 > kStaticScratchBytes - plan_bytes) return PIE_ENOMEM;
  out->plan = reinterpret_cast<int32_t*>(base);
  out->ws = reinterpret_cast<float*>(base + plan_bytes);
  out->ws_floats = ws_floats;
  out->n_counters = 2;          // one is used; two keep the item records 8-byte aligned
  out->lay_batch = batch;
  out->lay_max_blocks = max_blocks;
  return PIE_OK;
}

}  // namespace pie
