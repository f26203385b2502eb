// Small data-movement kernels: scatter of new K/V rows into the paged pool, whole-block
// gather / scatter between the pool and a contiguous staging buffer, and a plain
// streaming read used to measure what the memory system can deliver.
#include "kernels.h"

namespace heddle {

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// One workgroup per (pool block that receives new rows, kv head).  Trajectory b owns rows
// cu_rows[b] .. cu_rows[b+1] and write blocks cu_wblk[b] .. cu_wblk[b+1]; its row i goes to token
// position first_pos[b] + i.  K rows are copied as 16-byte pieces into the token-major K tile.
// V rows pass through LDS and leave transposed: a thread assembles the 8 consecutive tokens of
// one head-dim element and stores them as one 16-byte piece of the [d][16] V tile; where the new
// rows cover only part of those 8 slots the piece is read, merged and written back (the other
// slots belong to the same trajectory and nobody else writes this block during the call).
__device__ __forceinline__ void kv_write_block(const KvWriteLaunch& a, int wg) {
  constexpr int kMaxD = 128;
  __shared__ __attribute__((aligned(16))) uint16_t s_v[16][kMaxD + 8];
  const int wb = wg / a.n_kv_heads;
  const int h = wg - wb * a.n_kv_heads;
  int lo = 0, hi = a.B;                       // trajectory of this write block: last b with cu_wblk[b] <= wb
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (a.cu_wblk[mid] <= wb) lo = mid; else hi = mid;
  }
  const int b = lo;
  const int n_new = a.cu_rows[b + 1] - a.cu_rows[b];
  const int blk_in_traj = wb - a.cu_wblk[b];
  const int64_t row0 = a.cu_rows[b];
  const int first = a.first_pos[b];
  const int blk = first / 16 + blk_in_traj;                  // logical block
  const int t_lo = max(first, blk * 16), t_hi = min(first + n_new, blk * 16 + 16);
  const int s_lo = t_lo - blk * 16, s_hi = t_hi - blk * 16;  // slots [s_lo, s_hi) of the block are new
  const int64_t row_lo = row0 + (t_lo - first);              // source row of slot s_lo
  const int D = a.head_dim;
  const int pieces = D / 8;
  const int phys = a.block_ids[a.row_off[b] + blk];
  uint16_t* tile_k = a.pool + (static_cast<int64_t>(phys) * a.n_kv_heads + h) * 2 * 16 * D;
  uint16_t* tile_v = tile_k + 16 * D;

  for (int t = threadIdx.x; t < 16 * pieces; t += blockDim.x) {
    const int slot = t / pieces, c = t - slot * pieces;
    if (slot >= s_lo && slot < s_hi) {
      const int64_t src = ((row_lo + (slot - s_lo)) * a.n_kv_heads + h) * D + c * 8;
      *reinterpret_cast<u32x4*>(tile_k + slot * D + c * 8) = *reinterpret_cast<const u32x4*>(a.k + src);
      *reinterpret_cast<u32x4*>(&s_v[slot][c * 8]) = *reinterpret_cast<const u32x4*>(a.v + src);
    }
  }
  __syncthreads();
  for (int t = threadIdx.x; t < D * 2; t += blockDim.x) {
    const int e = t >> 1, half = t & 1;                       // head-dim element, slots 8*half .. 8*half+7
    const int lo8 = max(s_lo, 8 * half), hi8 = min(s_hi, 8 * half + 8);
    if (lo8 >= hi8) continue;
    u32x4* dst = reinterpret_cast<u32x4*>(tile_v + e * 16 + 8 * half);
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    if (hi8 - lo8 < 8) {
      const u32x4 old = *dst;
      w[0] = old.x, w[1] = old.y, w[2] = old.z, w[3] = old.w;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int slot = 8 * half + j;
      if (slot >= lo8 && slot < hi8) {
        const uint32_t x = s_v[slot][e];
        w[j >> 1] = (j & 1) ? (w[j >> 1] & 0x0000ffffu) | (x << 16) : (w[j >> 1] & 0xffff0000u) | x;
      }
    }
    *dst = u32x4{w[0], w[1], w[2], w[3]};
  }
}

__global__ __launch_bounds__(256) void kv_write_kernel(KvWriteLaunch a) { kv_write_block(a, blockIdx.x); }

// The row of a decode step: trajectory b stores row b of k / v at position first_pos[b].  One
// workgroup per (trajectory, kv head).  The K row goes out as 16-byte pieces; the V row is one
// 2-byte element per head-dim row of the transposed tile, stored as such (no read of the old
// piece).  The row itself and the table offset are fetched before the position is known.
__device__ __forceinline__ void kv_write_one_row(const KvWriteLaunch& a, int wg) {
  const int b = wg / a.n_kv_heads;
  const int h = wg - b * a.n_kv_heads;
  const int D = a.head_dim;
  const int tid = threadIdx.x;
  const int64_t src = (static_cast<int64_t>(b) * a.n_kv_heads + h) * D;
  u32x4 kpiece = {0u, 0u, 0u, 0u};
  uint16_t vel = 0;
  if (tid < D / 8) kpiece = *reinterpret_cast<const u32x4*>(a.k + src + tid * 8);
  if (tid < D) vel = a.v[src + tid];
  const int row_begin = a.row_off[b];
  const int first = a.first_pos[b];
  const int phys = a.block_ids[row_begin + first / 16];
  const int slot = first % 16;
  uint16_t* tile_k = a.pool + (static_cast<int64_t>(phys) * a.n_kv_heads + h) * 2 * 16 * D;
  uint16_t* tile_v = tile_k + 16 * D;
  if (tid < D / 8) *reinterpret_cast<u32x4*>(tile_k + slot * D + tid * 8) = kpiece;
  if (tid < D) tile_v[tid * 16 + slot] = vel;
}

// Gathers whole blocks of the pool into a contiguous staging buffer (PACK) or scatters them
// back under a list of physical blocks.  One workgroup moves one 4 KB slice of a block, one
// 16-byte non-temporal load and store per thread.
template <bool PACK>
__global__ __launch_bounds__(256) void kv_move_kernel(uint16_t* pool, uint16_t* staging, const int32_t* ids,
                                                       int32_t slices_per_block) {
  const int i = blockIdx.x / slices_per_block;   // index into ids and into staging
  const int slice = blockIdx.x - i * slices_per_block;
  const int64_t block_elems = static_cast<int64_t>(slices_per_block) * 2048;   // 4 KB = 2048 bf16
  const int64_t off = slice * 2048 + threadIdx.x * 8;
  u32x4* p = reinterpret_cast<u32x4*>(pool + static_cast<int64_t>(ids[i]) * block_elems + off);
  u32x4* s = reinterpret_cast<u32x4*>(staging + static_cast<int64_t>(i) * block_elems + off);
  if (PACK)
    __builtin_nontemporal_store(__builtin_nontemporal_load(p), s);
  else
    __builtin_nontemporal_store(__builtin_nontemporal_load(s), p);
}

// Block ids[n + i] of the pool becomes a copy of block ids[i]; same slicing as kv_move_kernel.
__global__ __launch_bounds__(256) void kv_copy_kernel(uint16_t* pool, const int32_t* ids, int32_t n,
                                                       int32_t slices_per_block) {
  const int i = blockIdx.x / slices_per_block;
  const int slice = blockIdx.x - i * slices_per_block;
  const int64_t block_elems = static_cast<int64_t>(slices_per_block) * 2048;
  const int64_t off = slice * 2048 + threadIdx.x * 8;
  const u32x4* s = reinterpret_cast<const u32x4*>(pool + static_cast<int64_t>(ids[i]) * block_elems + off);
  u32x4* d = reinterpret_cast<u32x4*>(pool + static_cast<int64_t>(ids[n + i]) * block_elems + off);
  __builtin_nontemporal_store(__builtin_nontemporal_load(s), d);
}

// The plan image of a call goes from the pinned staging buffer to device memory in this kernel
// rather than in a hipMemcpyAsync: between two kernels of a stream the runtime's copy of more than
// 16 KB costs about 17 us (it leaves the compute queue), this kernel 3-4 us for 20-64 KB.
__global__ __launch_bounds__(256) void plan_copy_kernel(const u32x4* src, u32x4* dst, uint32_t n_vec) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i < n_vec) dst[i] = src[i];
}

// The same copy and, in the workgroups behind it, the new K/V row of every trajectory of a decode
// step: one launch instead of two in front of the attention kernel.  The row writers read their
// trajectory's position from the pinned image (the device copy is being written meanwhile).
__global__ __launch_bounds__(256) void plan_copy_rows_kernel(const u32x4* src, u32x4* dst, uint32_t n_vec,
                                                              uint32_t copy_groups, KvWriteLaunch a) {
  if (blockIdx.x < copy_groups) {
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i < n_vec) dst[i] = src[i];
  } else {
    kv_write_one_row(a, static_cast<int>(blockIdx.x - copy_groups));
  }
}

constexpr int kStreamGroups = 2048;
constexpr int kStreamUnroll = 8;

// Contiguous 32 KB tiles (256 threads x 8 x 16 B) taken round robin by the workgroups, all
// eight loads of a thread in flight at once, non-temporal like the decode kernel's KV loads.
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* src, uint64_t n_vec, uint32_t* sink) {
  uint32_t x = 0;
  const uint64_t tile_vec = 256ull * kStreamUnroll;
  const uint64_t n_tiles = n_vec / tile_vec;
  for (uint64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
    const u32x4* p = src + t * tile_vec + threadIdx.x;
    u32x4 v[kStreamUnroll];
#pragma unroll
    for (int i = 0; i < kStreamUnroll; ++i) v[i] = __builtin_nontemporal_load(p + i * 256);
#pragma unroll
    for (int i = 0; i < kStreamUnroll; ++i) x ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
  }
  // remainder shorter than a tile
  for (uint64_t i = n_tiles * tile_vec + static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n_vec;
       i += static_cast<uint64_t>(gridDim.x) * blockDim.x) {
    const u32x4 v = src[i];
    x ^= v.x ^ v.y ^ v.z ^ v.w;
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x ^= __shfl_xor(x, off, 64);
  __shared__ uint32_t s[4];
  if ((threadIdx.x & 63) == 0) s[threadIdx.x >> 6] = x;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = s[0] ^ s[1] ^ s[2] ^ s[3];
}

}  // namespace

hipError_t launch_kv_write(const KvWriteLaunch& a, hipStream_t stream) {
  if (a.n_rows <= 0 || a.n_wblk <= 0) return hipSuccess;
  if (a.head_dim > 128 || a.one_row_each) return hipErrorInvalidValue;   // single rows go with the plan copy
  const dim3 grid(static_cast<unsigned>(a.n_wblk) * static_cast<unsigned>(a.n_kv_heads));
  hipLaunchKernelGGL(kv_write_kernel, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_kv_move(bool pack, void* pool, void* staging, const int32_t* ids, int32_t n, int64_t block_bytes,
                          hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  const int32_t slices = static_cast<int32_t>(block_bytes / 4096);
  const dim3 grid(static_cast<unsigned>(n) * static_cast<unsigned>(slices));
  if (pack)
    hipLaunchKernelGGL(kv_move_kernel<true>, grid, dim3(256), 0, stream, static_cast<uint16_t*>(pool),
                       static_cast<uint16_t*>(staging), ids, slices);
  else
    hipLaunchKernelGGL(kv_move_kernel<false>, grid, dim3(256), 0, stream, static_cast<uint16_t*>(pool),
                       static_cast<uint16_t*>(staging), ids, slices);
  return hipGetLastError();
}

hipError_t launch_kv_copy(void* pool, const int32_t* ids, int32_t n, int64_t block_bytes, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  const int32_t slices = static_cast<int32_t>(block_bytes / 4096);
  const dim3 grid(static_cast<unsigned>(n) * static_cast<unsigned>(slices));
  hipLaunchKernelGGL(kv_copy_kernel, grid, dim3(256), 0, stream, static_cast<uint16_t*>(pool), ids, n, slices);
  return hipGetLastError();
}

hipError_t launch_plan_copy(const void* src, void* dst, size_t n_vec, const KvWriteLaunch* rows, hipStream_t stream) {
  if (n_vec > 0x7fffffffu) return hipErrorInvalidValue;
  const unsigned copy_groups = static_cast<unsigned>((n_vec + 255) / 256);
  if (rows != nullptr && rows->n_wblk > 0) {
    if (!rows->one_row_each || rows->head_dim > 128) return hipErrorInvalidValue;
    const dim3 grid(copy_groups + static_cast<unsigned>(rows->n_wblk) * static_cast<unsigned>(rows->n_kv_heads));
    hipLaunchKernelGGL(plan_copy_rows_kernel, grid, dim3(256), 0, stream, static_cast<const u32x4*>(src),
                       static_cast<u32x4*>(dst), static_cast<uint32_t>(n_vec), copy_groups, *rows);
    return hipGetLastError();
  }
  if (n_vec == 0) return hipSuccess;
  hipLaunchKernelGGL(plan_copy_kernel, dim3(copy_groups), dim3(256), 0, stream, static_cast<const u32x4*>(src),
                     static_cast<u32x4*>(dst), static_cast<uint32_t>(n_vec));
  return hipGetLastError();
}

hipError_t launch_stream_read(const void* src, uint64_t bytes, uint32_t* sink, hipStream_t stream) {
  hipLaunchKernelGGL(stream_read_kernel, dim3(kStreamGroups), dim3(256), 0, stream,
                     static_cast<const u32x4*>(src), bytes / 16, sink);
  return hipGetLastError();
}

}  // namespace heddle
