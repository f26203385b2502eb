// Attention for tiles of at most 32 query rows (a few new tokens per trajectory times the G
// query heads of a kv head): the verify step of speculative decoding, the short tail of a
// chunk (paper Sec. 8).  Such a tile is bound by the K/V bytes it streams, not by matrix-core
// work, so it is organised like the decode kernel rather than like the 128-row append kernel:
//
//   * the four waves of a workgroup split the KEYS of the item, not the rows: wave w takes the
//     32-key tiles w, w+4, w+8, ... and keeps its own running (max, sum, O^T); the four states
//     are merged through LDS once, at the end;
//   * no barrier in the loop: nothing is shared between waves.
//       S^T = K Q^T  (v_mfma_f32_32x32x16_bf16, M = 32 keys, N = 32 rows).  Which key sits in row
//         m of the A tile is free: row m = 16u + 8a + 4b + c holds key 16u + 8b + 4a + c of the
//         tile.  With that choice accumulator register j of lane (n, hi) is key
//         16 (j/8) + 8 hi + j%8 of row n, i.e. registers 8u .. 8u+7 are already the B operand
//         P^T[8 hi + s][n] of block u with its keys in natural order.
//         The K tile (32 keys x 256 B) is fetched with coalesced 16-byte loads (a wave instruction
//         covers four whole key rows) and turned into operand layout (one key per lane) through
//         an 8 KB LDS area private to the wave: the LDS executes a wave's accesses in order, so
//         a compiler-level fence is all the synchronisation needed.  (Loading the operand layout
//         straight from memory, 16 bytes from each of 64 different lines per instruction, ran at
//         half the speed.)
//       O^T += V^T P^T: lane (m, hi) supplies V^T[32 mt + m][8 hi .. 8 hi + 7], a 16-byte piece
//         of the pool's transposed V tile straight from memory; a wave reads 1 KB contiguous per
//         (block, mt).
//   * the next 32-key tile (16 KB per wave) is loaded into registers while the current one is
//     multiplied; block ids come through the scalar cache.  Register pressure decides the rest:
//     a spilled register is reloaded through the vector memory counter and would make the wave
//     wait for its whole prefetch, so Q lives in LDS.
#include "kernels.h"

namespace heddle {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kBlockTokens = 16;
constexpr int kStepKeys = 64;           // granularity of item boundaries (AppendItemRec::step_begin)
constexpr int kTileKeys = 32;           // keys per MFMA tile of S^T
constexpr int kRows = 32;               // query rows (heads x chunk rows) per workgroup
constexpr float kLazyMaxSlack = 8.0f;   // log2 units

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

struct KvTile {            // one 32-key tile in flight: 16 x 16 B per lane
  u32x4 k[8];              // piece 64 i + lane of the K tile (key 4 i + lane / 16, d slice lane % 16)
  u32x4 v[2][4];           // [block of the tile][mt]: 8 keys of head-dim element 32 mt + m
};

__device__ __forceinline__ void wave_lds_fence() { asm volatile("" ::: "memory"); }

template <int D>
__global__ __launch_bounds__(256, 2) void narrow_attn_kernel(AppendLaunch a) {
  static_assert(D == 128, "operand mapping is written for head_dim 128");
  constexpr int NK = D / 16;
  constexpr int NMT = D / 32;
  const int G = a.n_q_heads / a.n_kv_heads;          // 1 .. 32
  const int RS = kRows / G;                          // chunk rows per workgroup tile (rounded down: rows past G*RS idle)
  constexpr int kTileElems = kBlockTokens * D;

  // merge buffer: [wave][mt][j][lane] accumulators, then [wave][3][lane] (max, rounded sum, sum).  During the
  // key loop the first 8 KB of a wave's accumulator area hold its K tile: key row t is 256 B,
  // its 16-byte piece c stored at slot c ^ (t & 15).
  __shared__ __attribute__((aligned(16))) float s_o[4][NMT][16][64];
  __shared__ float s_ml[4][3][64];

  const int item = blockIdx.x / a.n_kv_heads;
  const int h = blockIdx.x - item * a.n_kv_heads;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: tile indices stay scalar
  const int n = lane & 31;
  const int hi = lane >> 5;

  const AppendItemRec rec = a.items[item];
  const int b = rec.b;
  const int rows_n = rec.rows_n;
  const int key0 = rec.step_begin * kStepKeys;
  const int key_end = rec.key_end;
  const int L = a.ctx_len[b];
  const int kv_len = L + (a.cu_chunk[b + 1] - a.cu_chunk[b]);
  const int last_blk = (key_end - 1) / kBlockTokens;           // last logical block the item may touch
  typedef const __attribute__((address_space(4))) int32_t* const_ids_t;
  const const_ids_t ctable = (const_ids_t)(reinterpret_cast<uintptr_t>(a.block_ids + a.row_off[b]));

  // this lane's query row
  const int g = min(n / RS, G - 1);
  const int r_in_tile = n - g * RS;
  const bool row_valid = n < G * RS && r_in_tile < rows_n;
  const int chunk_row = rec.row0 + min(r_in_tile, rows_n - 1);
  const int64_t q_row = static_cast<int64_t>(a.cu_chunk[b]) + chunk_row;
  const int pos = L + chunk_row;                                // last key this row may see
  const int head = h * G + g;


  f32x16 o[NMT];
#pragma unroll
  for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
    for (int j = 0; j < 16; ++j) o[mt][j] = 0.0f;
  // l_sum: sum of the weights as they enter P.V (rounded to bf16), the output's denominator, so
  // that the weights stay normalised; l_exact: unrounded, for the log-sum-exp
  float m_ref = -INFINITY, l_sum = 0.0f, l_exact = 0.0f;

  const int64_t head_stride = 2 * kTileElems;
  const int64_t block_stride = static_cast<int64_t>(a.n_kv_heads) * head_stride;
  const uint16_t* pool_h = a.pool + h * head_stride;

  // key of the A-tile row this lane supplies: row m = 16u + 8a + 4b + c  <->  key 16u + 8b + 4a + c
  const int my_key = (n & 16) | ((n & 4) << 1) | ((n & 8) >> 1) | (n & 3);
  uint16_t* k_lds = reinterpret_cast<uint16_t*>(&s_o[wave][0][0][0]);

  // Q^T operand: B[k = d][n = row], 8 consecutive d per lane and step.  It is needed once per
  // tile only, so it waits in the second 8 KB of the wave's LDS area (piece kk of every lane
  // side by side) instead of occupying 32 registers.
  u32x4* q_lds = reinterpret_cast<u32x4*>(k_lds + kTileKeys * D) + lane;
  {
    const uint16_t* qp = a.q + (q_row * a.n_q_heads + head) * D + hi * 8;
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) q_lds[kk * 64] = *reinterpret_cast<const u32x4*>(qp + kk * 16);
  }
  const int ld_tok = lane >> 4, ld_slice = lane & 15;      // staging role within a group of 4 key rows

  const int n_tiles = (key_end - key0 + kTileKeys - 1) / kTileKeys;

  // physical ids of the two blocks of tile i (scalar loads; clamped so that a tile past the
  // item's end, which is never multiplied, still names a block of the trajectory)
  auto load_ids = [&](int i, int& id0, int& id1) {
    const int blk0 = (key0 + i * kTileKeys) / kBlockTokens;
    id0 = ctable[min(blk0, last_blk)];
    id1 = ctable[min(blk0 + 1, last_blk)];
  };
  auto load_tile = [&](int id0, int id1, KvTile& t) {
    const uint16_t* t0 = pool_h + static_cast<int64_t>(id0) * block_stride;
    const uint16_t* t1 = pool_h + static_cast<int64_t>(id1) * block_stride;
#pragma unroll
    for (int x = 0; x < 8; ++x) {                 // key 4 x + ld_tok of the tile: block x / 4, slot (4 x) % 16 + ld_tok
      const uint16_t* kp = (x >= 4 ? t1 : t0) + ((4 * x) % kBlockTokens + ld_tok) * D + ld_slice * 8;
      t.k[x] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kp));
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const uint16_t* vp = (u ? t1 : t0) + kTileElems + n * kBlockTokens + hi * 8;
#pragma unroll
      for (int mt = 0; mt < NMT; ++mt)
        t.v[u][mt] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vp + mt * 32 * kBlockTokens));
    }
  };

  auto compute_tile = [&](int i, KvTile& t) {
    const int T = key0 + i * kTileKeys;
    if (T + kTileKeys > kv_len) {                   // slots past the cache may hold NaN: clear their V
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int nv = kv_len - T - u * kBlockTokens - hi * 8;      // keys of this lane's piece that exist
        const uint32_t m0 = (0 < nv ? 0x0000ffffu : 0u) | (1 < nv ? 0xffff0000u : 0u);
        const uint32_t m1 = (2 < nv ? 0x0000ffffu : 0u) | (3 < nv ? 0xffff0000u : 0u);
        const uint32_t m2 = (4 < nv ? 0x0000ffffu : 0u) | (5 < nv ? 0xffff0000u : 0u);
        const uint32_t m3 = (6 < nv ? 0x0000ffffu : 0u) | (7 < nv ? 0xffff0000u : 0u);
#pragma unroll
        for (int mt = 0; mt < NMT; ++mt) {
          t.v[u][mt].x &= m0;
          t.v[u][mt].y &= m1;
          t.v[u][mt].z &= m2;
          t.v[u][mt].w &= m3;
        }
      }
    }
    // K tile: registers -> the wave's LDS area -> operand layout (this lane's key, slices 2 kk + hi)
    wave_lds_fence();
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      const int row = 4 * x + ld_tok;
      *reinterpret_cast<u32x4*>(k_lds + row * D + ((ld_slice ^ (row & 15)) * 8)) = t.k[x];
    }
    wave_lds_fence();
    f32x16 s;
#pragma unroll
    for (int j = 0; j < 16; ++j) s[j] = 0.0f;
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
      const int slot = (2 * kk + hi) ^ (my_key & 15);
      const bf16x8 ka = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(k_lds + my_key * D + slot * 8));
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, __builtin_bit_cast(bf16x8, q_lds[kk * 64]), s, 0, 0, 0);
    }
    wave_lds_fence();

    // register j is key T + 16 (j/8) + 8 hi + j%8 of this lane's row
    if (T + kTileKeys - 1 > L + rec.row0) {          // tile reaches the causal edge of some row
#pragma unroll
      for (int j = 0; j < 16; ++j)
        if (T + 16 * (j >> 3) + 8 * hi + (j & 7) > pos) s[j] = -INFINITY;
    }
    float mx = s[0];
#pragma unroll
    for (int j = 1; j < 16; ++j) mx = fmaxf(mx, s[j]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * a.scale_log2;
    if (__builtin_amdgcn_ballot_w64(mx > m_ref + kLazyMaxSlack) != 0) {
      const float m_new = fmaxf(m_ref, mx);
      const float shrink = m_new == -INFINITY ? 1.0f : __builtin_amdgcn_exp2f(m_ref - m_new);
      l_sum *= shrink;
      l_exact *= shrink;
#pragma unroll
      for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
        for (int j = 0; j < 16; ++j) o[mt][j] *= shrink;
      m_ref = m_new;
    }
    // a row that has seen no key yet keeps m_ref = -inf; its weights are exp2(-inf) = 0
    const float neg_m = m_ref == -INFINITY ? 0.0f : -m_ref;
    float p[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      p[j] = __builtin_amdgcn_exp2f(fmaf(s[j], a.scale_log2, neg_m));
      l_exact += p[j];
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      u32x4 w;
      w.x = pack_bf16(p[8 * u + 0], p[8 * u + 1]);
      w.y = pack_bf16(p[8 * u + 2], p[8 * u + 3]);
      w.z = pack_bf16(p[8 * u + 4], p[8 * u + 5]);
      w.w = pack_bf16(p[8 * u + 6], p[8 * u + 7]);
      l_sum += (__builtin_bit_cast(float, w.x << 16) + __builtin_bit_cast(float, w.x & 0xffff0000u)) +
               (__builtin_bit_cast(float, w.y << 16) + __builtin_bit_cast(float, w.y & 0xffff0000u)) +
               (__builtin_bit_cast(float, w.z << 16) + __builtin_bit_cast(float, w.z & 0xffff0000u)) +
               (__builtin_bit_cast(float, w.w << 16) + __builtin_bit_cast(float, w.w & 0xffff0000u));
      const bf16x8 pb = __builtin_bit_cast(bf16x8, w);
#pragma unroll
      for (int mt = 0; mt < NMT; ++mt)
        o[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, t.v[u][mt]), pb, o[mt], 0, 0, 0);
    }
  };

  // wave w owns tiles w, w + 4, ...; one tile is in flight while the previous one is multiplied
  KvTile cur, nxt;
  int i = wave, ida, idb;
  load_ids(i, ida, idb);
  if (i < n_tiles) load_tile(ida, idb, cur);
  load_ids(i + 4, ida, idb);
  while (i < n_tiles) {
    const int i_next = i + 4;
    if (i_next < n_tiles) load_tile(ida, idb, nxt);     // ids were requested one iteration ago
    load_ids(i_next + 4, ida, idb);
    compute_tile(i, cur);
    cur = nxt;
    i = i_next;
  }

  // ---- merge the four waves: wave w reduces head-dim rows 32 w .. 32 w + 31 of every query row
  wave_lds_fence();
  l_sum += __shfl_xor(l_sum, 32, 64);
  l_exact += __shfl_xor(l_exact, 32, 64);
#pragma unroll
  for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
    for (int j = 0; j < 16; ++j) s_o[wave][mt][j][lane] = o[mt][j];
  s_ml[wave][0][lane] = m_ref;
  s_ml[wave][1][lane] = l_sum;
  s_ml[wave][2][lane] = l_exact;
  __syncthreads();
  float mw[4], M = -INFINITY;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    mw[w] = s_ml[w][0][lane];
    M = fmaxf(M, mw[w]);
  }
  float l_all = 0.0f, l_all_exact = 0.0f, acc[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) acc[j] = 0.0f;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const float f = mw[w] == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f(mw[w] - M);
    l_all = fmaf(f, s_ml[w][1][lane], l_all);
    l_all_exact = fmaf(f, s_ml[w][2][lane], l_all_exact);
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = fmaf(f, s_o[w][wave][j][lane], acc[j]);
  }
  if (!row_valid) return;
  const int mt = wave;           // register j of this tile is head-dim element 32 mt + 8 (j/4) + 4 hi + j%4
  if (rec.nsplit > 1) {
    const int64_t slot = static_cast<int64_t>(rec.slot0 + r_in_tile * rec.nsplit) * a.n_q_heads + head;
    float* ap = a.part_acc + slot * D;
#pragma unroll
    for (int jq = 0; jq < 4; ++jq)
      *reinterpret_cast<float4*>(ap + mt * 32 + 8 * jq + 4 * hi) =
          float4{acc[4 * jq + 0], acc[4 * jq + 1], acc[4 * jq + 2], acc[4 * jq + 3]};
    if (wave == 0 && hi == 0) *reinterpret_cast<float4*>(a.part_ml + slot * 4) = float4{M, l_all, l_all_exact, 0.0f};
  } else {
    const float inv = 1.0f / l_all;
    uint16_t* op = a.out + (q_row * a.n_q_heads + head) * D;
#pragma unroll
    for (int jq = 0; jq < 4; ++jq) {
      u32x2 w;
      w.x = pack_bf16(acc[4 * jq + 0] * inv, acc[4 * jq + 1] * inv);
      w.y = pack_bf16(acc[4 * jq + 2] * inv, acc[4 * jq + 3] * inv);
      *reinterpret_cast<u32x2*>(op + mt * 32 + 8 * jq + 4 * hi) = w;
    }
    if (a.lse != nullptr && wave == 0 && hi == 0)
      a.lse[q_row * a.n_q_heads + head] = (M + __builtin_log2f(l_all_exact)) * 0.6931471805599453f;
  }
}

}  // namespace

int32_t narrow_tile_rows(int32_t group) { return kRows / group; }

hipError_t launch_narrow_attn(const AppendLaunch& a, hipStream_t stream) {
  if (a.n_items <= 0) return hipSuccess;
  const int G = a.n_q_heads / a.n_kv_heads;
  if (a.head_dim != 128 || G < 1 || G > kRows) return hipErrorInvalidValue;
  const dim3 grid(static_cast<unsigned>(a.n_items) * static_cast<unsigned>(a.n_kv_heads));
  hipLaunchKernelGGL((narrow_attn_kernel<128>), grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace heddle
