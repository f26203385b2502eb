// Causal chunked-append attention on the matrix cores (gfx950 MFMA).
//
// A tool-output chunk of C_b tokens is appended onto a trajectory's retained cache of L_b
// tokens (paper Sec. 2.1: each step of a trajectory continues from the previous context;
// Sec. 8 calls this tool-output prefill the dominant cost of prefill-heavy agents).  Chunk
// row i sits at position L_b + i and attends to positions 0 .. L_b + i.  The chunk's own
// K/V rows have been stored into the paged pool before this kernel runs.
//
// Work decomposition.  One workgroup (4 waves) owns a tile of 128 "rows": the G query heads
// of one kv head times 128/G consecutive chunk rows (rounded down: with G = 5, 25 rows per head and
// 3 idle rows), so the K/V bytes it reads are shared by all G heads.  G is a launch parameter, any
// value from 1 to 32.  Tiles arrive longest-first from the host plan.
//
// Transposed formulation.  Per 32 keys (two such tiles per 64-key main-loop step) the wave
// computes S^T = K Q^T (M = keys, N = query
// rows, contraction over d) and O^T += V^T P^T (M = head dim, N = query rows, contraction
// over keys) with v_mfma_f32_32x32x16_bf16.  Each lane then owns one query row (column
// n = lane % 32): its 16 accumulator registers of S^T are 16 keys of that row, so the row
// maximum and sum are register-local except for one exchange with lane ^ 32, and the
// C-layout of S^T is already the B-operand layout of P^T once the keys of a 16-key step are
// matched to the A-tile rows: the V planes are the natural halves {0-7 | 8-15} of the pool's rows
// (a 16-byte direct-to-LDS load cannot split them) and the K rows are assigned to A-tile rows in
// the matching permuted order.  P never moves between lanes.
//
// K tiles are token-major [16][d] and V tiles are transposed [d][16] in the pool, which is
// what the A operands want: 8 consecutive d of one key for K, 8 consecutive keys of one d
// for V.  Both are staged through LDS (XOR-swizzled K rows, V blocks as two planes of 8 keys,
// double buffer, one barrier per 64 keys) and shared by the four waves.  The next stage is
// filled by direct-to-LDS loads (global_load_lds_dwordx4) while the current one is multiplied:
// no staging registers, no LDS write instructions.
#include <type_traits>

#include "kernels.h"

namespace heddle {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kBlockTokens = 16;
constexpr int kChunkBlocks = 4;
constexpr int kChunkTokens = kChunkBlocks * kBlockTokens;   // keys per main-loop step
constexpr int kTileRows = 128;          // query rows (heads x chunk rows) per workgroup
constexpr int kMaxGroup = 32;           // query heads per kv head: a tile of the kernel for short-row tiles holds
                                        // one row of every head
constexpr float kLazyMaxSlack = 8.0f;   // log2 units

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;

// two floats -> packed bf16 pair (round to nearest even), one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// What a lane knows about its work item and its query row.
struct TileRow {
  int rows_n;          // rows of the tile that exist
  int extent;          // keys of the item, counted from its first key
  int kv_len;          // keys of the trajectory that exist, counted likewise (slots past it may hold anything)
  int edge;            // first position at which some row of the tile is masked
  int pos;             // last key this lane's row may see
  int part, nsplit;    // split-K partial slot of the row, parts of the tile
  int64_t q_row;       // row of q / out
  const int32_t* table;   // block ids of the item's first key onwards
  int head;            // query head of the row
  bool row_valid;      // the lane's row exists (else it mirrors the tile's last row and stores nothing)
};

// Decodes item `tile` for the lane whose query row is number n_global of the tile's 128:
// head g = n_global / R of the kv head's group, row n_global % R of the tile (R = 128 / G, rounded
// down: the last 128 - G*R rows of a tile carry nothing).
template <typename Launch>
__device__ __forceinline__ TileRow read_item(const Launch& a, int tile, int h, int n_global) {
  constexpr bool kGroup = std::is_same<Launch, GroupLaunch>::value;
  const int G = a.n_q_heads / a.n_kv_heads;
  const int R = kTileRows / G;
  const int g = min(n_global / R, G - 1);
  const int r_in_tile = n_global - g * R;
  TileRow t;
  t.head = h * G + g;
  t.part = 0;
  t.nsplit = 1;
  if constexpr (kGroup) {
    const GroupItemRec rec = a.items[tile];
    t.rows_n = rec.n_members;
    t.extent = (rec.blk_end - rec.blk_begin) * kBlockTokens;   // keys are counted from the item's first block
    t.kv_len = t.extent;
    t.table = a.block_ids + rec.table_off + rec.blk_begin;
    t.q_row = a.members[rec.member_off + min(r_in_tile, t.rows_n - 1)];
    t.pos = t.extent - 1;
    t.edge = t.extent - 1;
    t.part = a.trajs[t.q_row].part_off + rec.part;
  } else {
    const AppendItemRec rec = a.items[tile];
    const int b = rec.b;
    t.rows_n = rec.rows_n;
    const int key0 = rec.step_begin * kChunkTokens;   // keys are counted from the item's first step
    t.extent = rec.key_end - key0;
    const int L = a.ctx_len[b];
    t.kv_len = L + (a.cu_chunk[b + 1] - a.cu_chunk[b]) - key0;
    t.table = a.block_ids + a.row_off[b] + rec.step_begin * kChunkBlocks;
    const int chunk_row = rec.row0 + min(r_in_tile, t.rows_n - 1);
    t.q_row = static_cast<int64_t>(a.cu_chunk[b]) + chunk_row;
    t.pos = L + chunk_row - key0;
    t.edge = L + rec.row0 - key0;
    t.nsplit = rec.nsplit;
    t.part = rec.slot0 + min(r_in_tile, t.rows_n - 1) * t.nsplit;
  }
  t.row_valid = n_global < G * R && r_in_tile < t.rows_n;
  return t;
}

// Online softmax of one 64-key step.  s: the two 32-key tiles of S^T of this lane's row;
// key_of(u, j): index within the step of the key in register j of tile u (the kernels differ in
// the order of the A-tile rows).  masked: some row of the tile does not see all 64 keys.
// Moves the reference maximum lazily (slack 2^8), rescales o and l_sum when it moves, and returns
// p = 2^(s*scale - m) packed to bf16 in pw: registers 8v .. 8v+7 of tile u form pw[2u + v], the B
// operand of P^T for the 16-key block that the kernel pairs with them.
template <int NMT, typename KeyOf>
__device__ __forceinline__ void softmax_step(f32x16 (&s)[2], f32x16 (&o)[NMT], float& m_ref, float& l_sum,
                                             float scale_log2, bool masked, int t0, int pos, KeyOf key_of,
                                             u32x4 (&pw)[kChunkBlocks]) {
  if (masked) {
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int j = 0; j < 16; ++j)
        if (t0 + key_of(u, j) > pos) s[u][j] = -INFINITY;
  }
  float mx = s[0][0];
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int j = 0; j < 16; ++j) mx = fmaxf(mx, s[u][j]);
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale_log2;     // scale > 0: max commutes with it
  if (__builtin_amdgcn_ballot_w64(mx > m_ref + kLazyMaxSlack) != 0) {
    const float m_new = fmaxf(m_ref, mx);
    const float shrink = __builtin_amdgcn_exp2f(m_ref - m_new);
    l_sum *= shrink;
#pragma unroll
    for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
      for (int j = 0; j < 16; ++j) o[mt][j] *= shrink;
    m_ref = m_new;
  }
  const float neg_m = -m_ref;
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    float p[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      p[j] = __builtin_amdgcn_exp2f(fmaf(s[u][j], scale_log2, neg_m));
      l_sum += p[j];
    }
#pragma unroll
    for (int half_u = 0; half_u < 2; ++half_u) {
      u32x4 w;
      w.x = pack_bf16(p[8 * half_u + 0], p[8 * half_u + 1]);
      w.y = pack_bf16(p[8 * half_u + 2], p[8 * half_u + 3]);
      w.z = pack_bf16(p[8 * half_u + 4], p[8 * half_u + 5]);
      w.w = pack_bf16(p[8 * half_u + 6], p[8 * half_u + 7]);
      pw[2 * u + half_u] = w;
    }
  }
}

// Normalises and stores the lane's row (final bf16 output and log-sum-exp) or, for a part of a
// split tile and for shared-prefix items, its split-K partial.  Register j of tile mt of O^T is
// head-dim element mt*32 + 8*(j/4) + 4*hi + j%4.
template <int D, typename Launch>
__device__ __forceinline__ void store_row(const Launch& a, const TileRow& t, f32x16 (&o)[D / 32], float m_ref,
                                          float l_sum, int hi) {
  constexpr bool kGroup = std::is_same<Launch, GroupLaunch>::value;
  constexpr int NMT = D / 32;
  l_sum += __shfl_xor(l_sum, 32, 64);
  if (kGroup || t.nsplit > 1) {
    if (t.row_valid) {
      const int64_t slot = static_cast<int64_t>(t.part) * a.n_q_heads + t.head;
      float* ap = a.part_acc + slot * D;
#pragma unroll
      for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
        for (int jq = 0; jq < 4; ++jq)
          *reinterpret_cast<float4*>(ap + mt * 32 + 8 * jq + 4 * hi) =
              float4{o[mt][4 * jq + 0], o[mt][4 * jq + 1], o[mt][4 * jq + 2], o[mt][4 * jq + 3]};
      // the weights enter P.V rounded and the sum does not; the combine kernel takes the same sum
      // for the output's denominator and for the log-sum-exp of this part
      if (hi == 0) *reinterpret_cast<float4*>(a.part_ml + slot * 4) = float4{m_ref, l_sum, l_sum, 0.0f};
    }
  } else if constexpr (!kGroup) {
    if (t.row_valid) {
      const float inv = 1.0f / l_sum;
      uint16_t* op = a.out + (t.q_row * a.n_q_heads + t.head) * D;
#pragma unroll
      for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
        for (int jq = 0; jq < 4; ++jq) {
          u32x2 w;
          w.x = pack_bf16(o[mt][4 * jq + 0] * inv, o[mt][4 * jq + 1] * inv);
          w.y = pack_bf16(o[mt][4 * jq + 2] * inv, o[mt][4 * jq + 3] * inv);
          *reinterpret_cast<u32x2*>(op + mt * 32 + 8 * jq + 4 * hi) = w;
        }
      if (a.lse != nullptr && hi == 0)
        a.lse[t.q_row * a.n_q_heads + t.head] = (m_ref + __builtin_log2f(l_sum)) * 0.6931471805599453f;
    }
  }
}

// Launch = AppendLaunch: causal chunk rows of one trajectory against all their keys (final bf16
// output) or against one part of them (split-K partial, merged by decode_combine_kernel).
// Launch = GroupLaunch: the decode queries of the trajectories of a group against a range of the
// blocks they share (whole blocks, every key visible to every row), split-K partial output.
template <int D, typename Launch>
__global__ __launch_bounds__(256, 2) void append_dma_kernel(Launch a) {
  static_assert(D == 128 || D == 64, "staging roles and swizzle are written for head_dim 128 and 64");
  constexpr int NK = D / 16;             // MFMA steps over d for S^T
  constexpr int NMT = D / 32;            // 32-row tiles of O^T over d
  constexpr int kTileElems = kBlockTokens * D;
  constexpr int kStageK = kChunkTokens * D;            // elements of K per LDS stage
  constexpr int kStageV = kChunkBlocks * kTileElems;   // elements of V per LDS stage
  constexpr int kVPlane = D * 8;                       // elements of one 8-key plane of a V block

  // Two stages of K and of V, each an LDS object of its own: the compiler then knows that a
  // direct-to-LDS load into one stage does not alias the operand reads of the other and does not
  // make those reads wait for it.  K rows are 2 D bytes = D/8 slots of 16 B (16 at d = 128); slot c
  // of key row t sits at slot c ^ (t & (D/8 - 1)), so that the 32 lanes reading the same d-slice of
  // 32 different keys spread over the banks.  A V block is two planes of [d][8 keys] (plane 0 keys
  // 0-7, plane 1 keys 8-15): the 16 lanes an LDS read serves per cycle, consecutive head-dim rows of
  // one plane, fall into 16 different bank groups.
  __shared__ __attribute__((aligned(16))) uint16_t s_k0[kStageK];
  __shared__ __attribute__((aligned(16))) uint16_t s_k1[kStageK];
  __shared__ __attribute__((aligned(16))) uint16_t s_v0[kStageV];
  __shared__ __attribute__((aligned(16))) uint16_t s_v1[kStageV];

  const int tile = blockIdx.x / a.n_kv_heads;
  const int h = blockIdx.x - tile * a.n_kv_heads;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int n = lane & 31;               // query row (column of S^T / O^T) within the wave
  const int hi = lane >> 5;

  // this lane's work item and query row (row wave*32 + n of the tile's 128)
  const TileRow tr = read_item(a, tile, h, wave * 32 + n);
  const int extent = tr.extent, kv_len = tr.kv_len, edge = tr.edge, pos = tr.pos;
  const int32_t* const table = tr.table;

  // Q^T operand: B[k = d][n = row], 8 consecutive d per lane and step
  bf16x8 qb[NK];
  {
    const uint16_t* qp = a.q + (tr.q_row * a.n_q_heads + tr.head) * D + hi * 8;
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) qb[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qp + kk * 16));
  }

  f32x16 o[NMT];
#pragma unroll
  for (int mt = 0; mt < NMT; ++mt)
#pragma unroll
    for (int j = 0; j < 16; ++j) o[mt][j] = 0.0f;
  float m_ref = -INFINITY, l_sum = 0.0f;

  const int64_t head_stride = 2 * kTileElems;
  const int64_t block_stride = static_cast<int64_t>(a.n_kv_heads) * head_stride;
  const int n_blocks_needed = (extent + kBlockTokens - 1) / kBlockTokens;
  const int n_chunks = (extent + kChunkTokens - 1) / kChunkTokens;

  // Staging.  A wave-level direct-to-LDS load moves 64 x 16 B from per-lane global addresses to
  // 1 KB of consecutive LDS: the swizzle of the K rows is therefore applied on the global side.
  // A stage of K is D/8 such loads (kRowsPerLoad key rows each), a stage of V as many (one plane of
  // 64 head-dim rows of one block each); a wave issues every fourth of them, D/32 of K and of V:
  //   K load 4k + w: key rows kRowsPerLoad (4k + w) .. of the chunk: lane i -> row i / kSlots of them,
  //      LDS slot i % kSlots, which holds the row's piece (i % kSlots) ^ (row & (kSlots - 1))
  //   V load 4k + w: block (4k + w) / kLoadsPerBlock, plane and 64-row group from (4k + w) % kLoadsPerBlock
  // d = 128: a wave's k-th loads belong to block k; d = 64: to block 2k + w/2 (uniform per wave).
  constexpr int kSlots = D / 8;                       // 16-byte pieces of a K row
  constexpr int kRowsPerLoad = 64 / kSlots;           // 4 or 8
  constexpr int kLoadsPerWave = D / 32;               // of K, and of V, per stage
  constexpr int kLoadsPerBlock = D / 32;              // of V (two planes x D/64 groups of 64 rows); of K: 16 / kRowsPerLoad
  const int wv = __builtin_amdgcn_readfirstlane(wave);
  const int k_row_in = (kRowsPerLoad * wv) % kBlockTokens + lane / kSlots;       // row within its block
  const uint32_t k_goff =
      static_cast<uint32_t>(k_row_in * D + (((lane % kSlots) ^ (k_row_in & (kSlots - 1))) * 8)) * 2u;
  const int v_within = wv % kLoadsPerBlock, v_plane = v_within & 1, v_group = v_within >> 1;
  const uint32_t v_goff = static_cast<uint32_t>(kTileElems + (64 * v_group + lane) * kBlockTokens + v_plane * 8) * 2u;
  // block of this wave's k-th load (the same for K and V) and the LDS offsets of the loads, in elements
  auto load_block = [&](int k) { return D == 128 ? k : 2 * k + (wv >> 1); };
  auto k_loff = [&](int k) { return kRowsPerLoad * (4 * k + wv) * D; };
  auto v_loff = [&](int k) { return load_block(k) * kTileElems + v_plane * kVPlane + v_group * 64 * 8; };
  // the item's last chunk may hold slots past the cache, whose V must not reach the matrix cores
  // (0 x NaN): that chunk's V goes through registers, is cleared there and stored with ds_write:
  // piece tid + 256 k of the chunk's 4 x 2 D pieces, i.e. block (tid + 256 k) / (2 D), head-dim row
  // and key half from the remainder
  constexpr int kPiecesPerBlock = 2 * D;
  constexpr int kPiecesPerThread = kChunkBlocks * kPiecesPerBlock / 256;           // 4 or 2
  const int v_row = (tid % kPiecesPerBlock) >> 1, v_half = tid & 1;
  const uint32_t v_piece = static_cast<uint32_t>(kTileElems + v_row * kBlockTokens + v_half * 8) * 2u;

  typedef const __attribute__((address_space(4))) int32_t* const_ids_t;
  const const_ids_t ctable = (const_ids_t)(reinterpret_cast<uintptr_t>(table));
  int ids[kChunkBlocks];
  auto load_ids = [&](int c) {
#pragma unroll
    for (int x = 0; x < kChunkBlocks; ++x) ids[x] = ctable[min(kChunkBlocks * c + x, n_blocks_needed - 1)];
  };
  typedef int32_t ids4_t __attribute__((ext_vector_type(4), aligned(4)));
  typedef const __attribute__((address_space(4))) ids4_t* const_ids4_t;
  auto load_ids_whole = [&](int c) {                  // a chunk whose four blocks all lie inside the item
    const ids4_t v = *(const_ids4_t)(ctable + kChunkBlocks * c);
    ids[0] = v.x, ids[1] = v.y, ids[2] = v.z, ids[3] = v.w;
  };

  const char* pool_h = reinterpret_cast<const char*>(a.pool + h * head_stride);
  const uint32_t block_bytes = static_cast<uint32_t>(block_stride * 2);   // at most 32 kv heads x 8 KB
  typedef const __attribute__((address_space(1))) char* gptr_t;
  typedef const __attribute__((address_space(1))) void* gvoid_t;
  typedef const __attribute__((address_space(1))) u32x4* gvec_t;
  typedef __attribute__((address_space(3))) void* lvoid_t;

  // block id number x of the chunk in `ids`, x uniform per wave (a constant at d = 128)
  auto id_of = [&](int x) { return x == 0 ? ids[0] : x == 1 ? ids[1] : x == 2 ? ids[2] : ids[3]; };
  auto block_base = [&](int x) {
    uint64_t base = reinterpret_cast<uint64_t>(pool_h) + static_cast<uint64_t>(static_cast<uint32_t>(id_of(x))) * block_bytes;
    asm("" : "+s"(base));                 // 32 x 32 -> 64 bits in scalar registers, next to the load
    return reinterpret_cast<gptr_t>(base);
  };
  // stages chunk cn (whose block ids are in `ids`) into stage STN; v_by_regs: see above
  auto stage_chunk = [&](int cn, auto stn, bool v_by_regs) {
    constexpr int STN = decltype(stn)::value;
    uint16_t* const kdst = STN ? s_k1 : s_k0;
    uint16_t* const vdst = STN ? s_v1 : s_v0;
    gptr_t base[kLoadsPerWave];
#pragma unroll
    for (int k = 0; k < kLoadsPerWave; ++k) {
      base[k] = block_base(load_block(k));
      __builtin_amdgcn_global_load_lds((gvoid_t)(base[k] + k_goff), (lvoid_t)(kdst + k_loff(k)), 16, 0, 0);
    }
    if (!v_by_regs) {
#pragma unroll
      for (int k = 0; k < kLoadsPerWave; ++k)
        __builtin_amdgcn_global_load_lds((gvoid_t)(base[k] + v_goff), (lvoid_t)(vdst + v_loff(k)), 16, 0, 0);
    } else {
#pragma unroll
      for (int k = 0; k < kPiecesPerThread; ++k) {
        const int x = load_block(k);                           // = (tid + 256 k) / kPiecesPerBlock, uniform per wave
        const int blk = kChunkBlocks * cn + x;
        u32x4 vv = *reinterpret_cast<gvec_t>(block_base(x) + v_piece);
        const int nv = kv_len - blk * kBlockTokens - v_half * 8;   // keys of this piece that exist; the rest may be NaN
        vv.x &= (0 < nv ? 0x0000ffffu : 0u) | (1 < nv ? 0xffff0000u : 0u);
        vv.y &= (2 < nv ? 0x0000ffffu : 0u) | (3 < nv ? 0xffff0000u : 0u);
        vv.z &= (4 < nv ? 0x0000ffffu : 0u) | (5 < nv ? 0xffff0000u : 0u);
        vv.w &= (6 < nv ? 0x0000ffffu : 0u) | (7 < nv ? 0xffff0000u : 0u);
        *reinterpret_cast<u32x4*>(vdst + x * kTileElems + v_half * kVPlane + v_row * 8) = vv;
      }
    }
  };

  // key of the A-tile row this lane supplies: row 16u + 8a + 4b + c of a 32-key tile holds key
  // 16u + 8b + 4a + c, so that accumulator registers 8v .. 8v + 7 of S^T are the B operand of P^T
  // for block v of the tile with its keys 8 hi .. 8 hi + 7 in natural order (the order of a V plane)
  const int my_key = (n & 16) | ((n & 4) << 1) | ((n & 8) >> 1) | (n & 3);

  load_ids(0);
  stage_chunk(0, std::integral_constant<int, 0>{}, n_chunks == 1);
  load_ids(1);

  auto step = [&](int c, auto interior, auto stc) {
    constexpr bool kInterior = decltype(interior)::value;
    constexpr int ST = decltype(stc)::value;
    const uint16_t* const ks = ST ? s_k1 : s_k0;
    const uint16_t* const vs = ST ? s_v1 : s_v0;
    // this wave's direct-to-LDS loads of stage ST have landed (the barrier alone does not wait for
    // them); behind the barrier stage ST is complete and nobody reads the other stage any more
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (kInterior) stage_chunk(c + 1, std::integral_constant<int, ST ^ 1>{}, false);
    else if (c + 1 < n_chunks) stage_chunk(c + 1, std::integral_constant<int, ST ^ 1>{}, c + 2 == n_chunks);
    if (kInterior) load_ids_whole(c + 2);
    else load_ids(c + 2);                  // clamped to the tile's last block

    const int t0 = c * kChunkTokens;

    // ---- S^T = K Q^T : two tiles of 32 keys x 32 rows
    f32x16 s[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
      for (int j = 0; j < 16; ++j) s[u][j] = 0.0f;
      const int row = 32 * u + my_key;
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) {
        const int slot = (2 * kk + hi) ^ (my_key & (kSlots - 1));
        const bf16x8 ka = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(&ks[row * D + slot * 8]));
        s[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qb[kk], s[u], 0, 0, 0);
      }
    }

    // register j of tile u is key t0 + 32u + 16*(j/8) + 8*hi + j%8 of this lane's row
    u32x4 pw[kChunkBlocks];
    softmax_step<NMT>(s, o, m_ref, l_sum, a.scale_log2, !kInterior && t0 + kChunkTokens - 1 > edge, t0, pos,
                      [hi](int u, int j) { return 32 * u + 16 * (j >> 3) + 8 * hi + (j & 7); }, pw);

    // ---- O^T += V^T P^T : one 16-key step per block, NMT tiles of 32 head-dim rows
#pragma unroll
    for (int x = 0; x < kChunkBlocks; ++x) {
      const bf16x8 pb = __builtin_bit_cast(bf16x8, pw[x]);
#pragma unroll
      for (int mt = 0; mt < NMT; ++mt) {
        const bf16x8 va = __builtin_bit_cast(
            bf16x8, *reinterpret_cast<const u32x4*>(&vs[x * kTileElems + hi * kVPlane + (mt * 32 + n) * 8]));
        o[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb, o[mt], 0, 0, 0);
      }
    }
  };

  // Steps [0, n_interior) are interior: no mask, and the chunks they stage (c + 1) and look up
  // (c + 2) are whole chunks of the item before its last one.  The loop advances two steps at a
  // time so that the stage of a step is known at compile time.
  const int n_interior = max(0, min(n_chunks - 3, (edge + 1) / kChunkTokens));
  int c = 0;
  for (; c + 1 < n_interior; c += 2) {
    step(c, std::true_type{}, std::integral_constant<int, 0>{});
    step(c + 1, std::true_type{}, std::integral_constant<int, 1>{});
  }
  for (; c < n_chunks; c += 2) {
    step(c, std::false_type{}, std::integral_constant<int, 0>{});
    if (c + 1 < n_chunks) step(c + 1, std::false_type{}, std::integral_constant<int, 1>{});
  }

  store_row<D>(a, tr, o, m_ref, l_sum, hi);
}

template <typename Launch>
hipError_t launch_t(const Launch& a, hipStream_t stream) {
  const dim3 grid(static_cast<unsigned>(a.n_items) * static_cast<unsigned>(a.n_kv_heads));
  if (a.head_dim == 128)
    hipLaunchKernelGGL((append_dma_kernel<128, Launch>), grid, dim3(256), 0, stream, a);
  else
    hipLaunchKernelGGL((append_dma_kernel<64, Launch>), grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace

bool append_shape_supported(int32_t group, int32_t head_dim) {
  return (head_dim == 128 || head_dim == 64) && group >= 1 && group <= kMaxGroup;
}

int32_t append_tile_rows(int32_t group) { return kTileRows / group; }

hipError_t launch_append_attn(const AppendLaunch& a, hipStream_t stream) {
  if (a.n_items <= 0) return hipSuccess;
  if (!append_shape_supported(a.n_q_heads / a.n_kv_heads, a.head_dim)) return hipErrorInvalidValue;
  return launch_t(a, stream);
}

hipError_t launch_group_attn(const GroupLaunch& a, hipStream_t stream) {
  if (a.n_items <= 0) return hipSuccess;
  if (!append_shape_supported(a.n_q_heads / a.n_kv_heads, a.head_dim)) return hipErrorInvalidValue;
  return launch_t(a, stream);
}

}  // namespace heddle
