// Small data-movement kernels: scatter of new K/V rows into the paged pool, whole-block
// gather / scatter between the pool and a contiguous staging buffer, and a plain
// streaming read used to measure what the memory system can deliver.
#include "kernels.h"

namespace heddle {

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// One workgroup per new token row; thread t moves one 8-element piece of K (one 16-byte
// store into the token-major K tile) and of V (eight 2-byte stores into the transposed V
// tile, where the 16 tokens of a head-dim element are contiguous).
// Row i of trajectory b (rows cu_rows[b] .. cu_rows[b+1]) goes to position first_pos[b] + i.
__global__ __launch_bounds__(256) void kv_write_kernel(KvWriteLaunch a) {
  const int row = blockIdx.x;
  // trajectory of this row: last b with cu_rows[b] <= row
  int lo = 0, hi = a.B;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (a.cu_rows[mid] <= row) lo = mid; else hi = mid;
  }
  const int b = lo;
  const int pos = a.first_pos[b] + (row - a.cu_rows[b]);
  const int phys = a.block_ids[a.row_off[b] + pos / 16];
  const int slot = pos % 16;
  const int D = a.head_dim;
  const int pieces_per_head = D / 8;
  const int n_pieces = a.n_kv_heads * pieces_per_head;
  for (int t = threadIdx.x; t < n_pieces; t += blockDim.x) {
    const int h = t / pieces_per_head;
    const int c = t - h * pieces_per_head;
    const int64_t src = (static_cast<int64_t>(row) * a.n_kv_heads + h) * D + c * 8;
    const int64_t tile_k = (static_cast<int64_t>(phys) * a.n_kv_heads + h) * 2 * 16 * D;
    const int64_t tile_v = tile_k + 16 * D;
    *reinterpret_cast<u32x4*>(a.pool + tile_k + slot * D + c * 8) = *reinterpret_cast<const u32x4*>(a.k + src);
    const u32x4 vv = *reinterpret_cast<const u32x4*>(a.v + src);
    const uint32_t w[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint16_t x = static_cast<uint16_t>(e & 1 ? w[e >> 1] >> 16 : w[e >> 1] & 0xffffu);
      a.pool[tile_v + static_cast<int64_t>(c * 8 + e) * 16 + slot] = x;
    }
  }
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
  if (a.n_rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(kv_write_kernel, dim3(static_cast<unsigned>(a.n_rows)), dim3(256), 0, stream, a);
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

hipError_t launch_stream_read(const void* src, uint64_t bytes, uint32_t* sink, hipStream_t stream) {
  hipLaunchKernelGGL(stream_read_kernel, dim3(kStreamGroups), dim3(256), 0, stream,
                     static_cast<const u32x4*>(src), bytes / 16, sink);
  return hipGetLastError();
}

}  // namespace heddle
