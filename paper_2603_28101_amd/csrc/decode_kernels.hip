// Split-K decode attention over a paged KV pool, and the log-sum-exp merge of the parts of
// trajectories that were split (an unsplit trajectory is finished by its only item).
//
// One query token per trajectory attends to its whole retained context (paper Sec. 2.1:
// generation steps of a multi-step trajectory; Sec. 4.2: the KV cache persists between
// steps).  Contexts are long-tailed (Sec. 2.2), so the host plan cuts long ones into items;
// a workgroup handles one (item, kv head) and all G query heads that share that kv head.
//
// This is a streaming kernel: every K and V byte is read once, straight from HBM into
// registers in fully coalesced 1 KB wave loads, and used by G heads.  No matrix cores.
// The loads are non-temporal: the data is never reused, and on this chip a read stream
// that bypasses cache retention runs about 12 % faster than one that does not.
//
// Per 16-token block and wave (wave64):
//   Q.K   The K tile is token-major [16][d]; a row of d bf16 is covered by d/8 lanes holding
//         8 elements (16 bytes) each.  Every lane forms G partial dot products per load with
//         packed-bf16 dot instructions.  The partials of a row are then summed with a
//         reduce-scatter over its lanes (DPP adds): each step halves the number of values a
//         lane carries, so a lane ends with the complete logit of one (token, head) pair (two
//         for G = 8) instead of every lane ending with all of them.
//   softmax  runs once per (token, head), in base 2, against a lazily updated reference
//         maximum per head: the reference moves (and accumulators are rescaled) only when a
//         logit exceeds it by more than 2^8, which is rare after the first blocks.
//   P.V   The V tile is stored transposed, [d][16]: a lane's 16 bytes are 8 consecutive tokens
//         of one head-dim element, so P.V is again packed-bf16 dot products, acc[g][e] +=
//         p[g][t..t+1] . v[e][t..t+1], with p rounded to bf16 and passed between lanes through
//         a 32-byte-per-head LDS row private to the wave.  The softmax denominator used for
//         the output is the sum of the same rounded p (so the weights stay normalised); the
//         log-sum-exp output uses the unrounded sum.
#include "kernels.h"

namespace heddle {

namespace {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kBlockTokens = 16;
constexpr int kWavesPerGroup = 4;
constexpr int kSameHeadStride = 4;      // lanes l and l + 4k carry the same query head(s)
constexpr float kLazyMaxSlack = 8.0f;   // log2 units

// Lanes of one wave exchange values through LDS without a hardware barrier: the LDS executes
// a wave's instructions in order, so a read issued after a write sees it.  The compiler must
// still be told that memory may have changed under it (other lanes wrote), or it forwards a
// lane's own store into its later load and hoists loads above stores of other lanes.
__device__ __forceinline__ void wave_lds_fence() { asm volatile("" ::: "memory"); }

template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true);
  return x + __builtin_bit_cast(float, moved);
}

constexpr int kDppXor1 = 0xB1;          // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;          // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;   // lane i <- lane 7 - i within each 8 lanes
constexpr int kDppMirror = 0x140;       // lane i <- lane 15 - i within each 16 lanes

// One halving step of the reduce-scatter across lane pairs (i, 15 - i) [FULL] or (i, 7 - i)
// within 8 lanes [!FULL].  The lane of a pair that sits in the lower half keeps lo, the other
// keeps hi; both receive own + partner for the value they keep.  Two DPP adds with
// complementary bank masks write the two halves of the same destination register.  The
// leading s_nop covers the wait states a DPP read needs after the dot instructions that
// produced the inputs; inline assembly is not covered by the compiler's hazard handling.
template <bool FULL>
__device__ __forceinline__ void pair_reduce4(float& o0, float& o1, float& o2, float& o3, float l0, float l1,
                                             float l2, float l3, float h0, float h1, float h2, float h3) {
  if constexpr (FULL) {
    asm("s_nop 4\n\t"
        "v_add_f32_dpp %0, %4, %4 row_mirror row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %0, %8, %8 row_mirror row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %1, %5, %5 row_mirror row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %1, %9, %9 row_mirror row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %2, %6, %6 row_mirror row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %2, %10, %10 row_mirror row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %3, %7, %7 row_mirror row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %3, %11, %11 row_mirror row_mask:0xf bank_mask:0xc\n\t"
        "s_nop 1"
        : "=&v"(o0), "=&v"(o1), "=&v"(o2), "=&v"(o3)
        : "v"(l0), "v"(l1), "v"(l2), "v"(l3), "v"(h0), "v"(h1), "v"(h2), "v"(h3));
  } else {
    asm("s_nop 4\n\t"
        "v_add_f32_dpp %0, %4, %4 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %0, %8, %8 row_half_mirror row_mask:0xf bank_mask:0xa\n\t"
        "v_add_f32_dpp %1, %5, %5 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %1, %9, %9 row_half_mirror row_mask:0xf bank_mask:0xa\n\t"
        "v_add_f32_dpp %2, %6, %6 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %2, %10, %10 row_half_mirror row_mask:0xf bank_mask:0xa\n\t"
        "v_add_f32_dpp %3, %7, %7 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %3, %11, %11 row_half_mirror row_mask:0xf bank_mask:0xa\n\t"
        "s_nop 1"
        : "=&v"(o0), "=&v"(o1), "=&v"(o2), "=&v"(o3)
        : "v"(l0), "v"(l1), "v"(l2), "v"(l3), "v"(h0), "v"(h1), "v"(h2), "v"(h3));
  }
}

template <bool FULL>
__device__ __forceinline__ void pair_reduce1(float& o, float lo, float hi) {
  if constexpr (FULL) {
    asm("s_nop 4\n\t"
        "v_add_f32_dpp %0, %1, %1 row_mirror row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %0, %2, %2 row_mirror row_mask:0xf bank_mask:0xc\n\t"
        "s_nop 1"
        : "=&v"(o)
        : "v"(lo), "v"(hi));
  } else {
    asm("s_nop 4\n\t"
        "v_add_f32_dpp %0, %1, %1 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %0, %2, %2 row_half_mirror row_mask:0xf bank_mask:0xa\n\t"
        "s_nop 1"
        : "=&v"(o)
        : "v"(lo), "v"(hi));
  }
}

constexpr int half_or_one(int n) { return n > 1 ? n / 2 : 1; }

// in[CNT] -> out[max(CNT/2,1)] across mirror pairs; with a single value left it is summed
// into both lanes instead (all-reduce step).
template <bool FULL, int CNT>
__device__ __forceinline__ void level_mirror(const float (&in)[CNT], float (&out)[half_or_one(CNT)]) {
  if constexpr (CNT == 1) {
    out[0] = dpp_add<FULL ? kDppMirror : kDppHalfMirror>(in[0]);
  } else {
    constexpr int H = CNT / 2;
    if constexpr (H % 4 == 0) {
#pragma unroll
      for (int k = 0; k < H; k += 4)
        pair_reduce4<FULL>(out[k], out[k + 1], out[k + 2], out[k + 3], in[k], in[k + 1], in[k + 2], in[k + 3],
                           in[H + k], in[H + k + 1], in[H + k + 2], in[H + k + 3]);
    } else {
#pragma unroll
      for (int k = 0; k < H; ++k) pair_reduce1<FULL>(out[k], in[k], in[H + k]);
    }
  }
}

// Same halving across lane pairs (i, i ^ 2) or (i, i ^ 1); `upper` tells whether this lane is
// the one of its pair that keeps the upper half.
template <int CTRL, int CNT>
__device__ __forceinline__ void level_quad(const float (&in)[CNT], float (&out)[half_or_one(CNT)], bool upper) {
  if constexpr (CNT == 1) {
    out[0] = dpp_add<CTRL>(in[0]);
  } else {
    constexpr int H = CNT / 2;
#pragma unroll
    for (int k = 0; k < H; ++k) {
      const float lo = dpp_add<CTRL>(in[k]);
      const float hi = dpp_add<CTRL>(in[H + k]);
      out[k] = upper ? hi : lo;
    }
  }
}

// Sums x[n] over the LPR lanes of a token row.  With N >= LPR values per lane, lane c of the
// row ends with the N/LPR complete sums of indices c*N/LPR ...; with fewer, index c / (LPR/N)
// is replicated over LPR/N neighbouring lanes.
template <int LPR, int N>
__device__ __forceinline__ void row_reduce_scatter(const float (&x)[N], float (&y)[(N >= LPR) ? N / LPR : 1], int lane) {
  constexpr int C1 = (LPR == 16) ? half_or_one(N) : N;
  constexpr int C2 = half_or_one(C1);
  constexpr int C3 = half_or_one(C2);
  constexpr int C4 = half_or_one(C3);
  static_assert(C4 == ((N >= LPR) ? N / LPR : 1), "level sizes");
  float a[C1], b[C2], c[C3];
  if constexpr (LPR == 16) {
    level_mirror<true, N>(x, a);
  } else {
#pragma unroll
    for (int k = 0; k < N; ++k) a[k] = x[k];
  }
  level_mirror<false, C1>(a, b);
  level_quad<kDppXor2, C2>(b, c, (lane & 2) != 0);
  level_quad<kDppXor1, C3>(c, y, (lane & 1) != 0);
}

__device__ __forceinline__ float same_head_max(float x) {
#pragma unroll
  for (int off = kSameHeadStride; off < 64; off <<= 1) x = fmaxf(x, __shfl_xor(x, off, 64));
  return x;
}

__device__ __forceinline__ float same_head_sum(float x) {
#pragma unroll
  for (int off = kSameHeadStride; off < 64; off <<= 1) x += __shfl_xor(x, off, 64);
  return x;
}

// The packed operands go through a by-value helper: a bit cast applied directly to a
// vector element (v.y) reads element 0 with this compiler.
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}

__device__ __forceinline__ float dot8(const u32x4& a, const u32x4& b, float s) {
  s = dot2(a.x, b.x, s);
  s = dot2(a.y, b.y, s);
  s = dot2(a.z, b.z, s);
  s = dot2(a.w, b.w, s);
  return s;
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

// G: query heads per kv head.  D: head dim.  PF: KV blocks kept in flight per wave.
template <int G, int D, int PF>
__global__ __launch_bounds__(kWavesPerGroup * 64, 2) void decode_splitk_kernel(DecodeLaunch a) {
  constexpr int LPR = D / 8;                // lanes per K row
  constexpr int TPI = 64 / LPR;             // K rows (tokens) per wave load instruction
  constexpr int NI = kBlockTokens / TPI;    // load instructions per K tile (and per V tile)
  constexpr int N = G * NI;                 // partial logits per lane and block
  constexpr int VPL = (N >= LPR) ? N / LPR : 1;   // complete logits per lane after the reduce
  constexpr int REP = (N >= LPR) ? 1 : LPR / N;   // lanes that share one logit otherwise
  constexpr int kTileElems = kBlockTokens * D;
  static_assert(LPR / NI == kSameHeadStride, "lanes that share a head are 4 apart");

  const int item = blockIdx.x / a.n_kv_heads;
  const int h = blockIdx.x - item * a.n_kv_heads;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = lane / LPR;                 // K: token row within a load instruction
  const int c = lane - r * LPR;             // K: 8-element slice of the head dim
  const int half = lane & 1;                // V: which 8 of the block's 16 tokens
  // (token, head) of this lane's complete logits: index n = i*G + g over (load i, head g)
  const int n0 = (N >= LPR) ? c * VPL : c / REP;
  const int my_tok = (n0 / G) * TPI + r;    // token within the block
  const int my_g0 = n0 % G;                 // first (or only) head; the second is my_g0 + 1

  const DecodeItemRec rec = a.items[item];
  const int b = rec.b;
  const int blk_begin = rec.blk_begin;
  const int blk_end = rec.blk_end;
  const int len = rec.len;
  const int32_t* table = a.block_ids + rec.table_off;
  const int slot = rec.slot;

  // each wave streams a contiguous quarter of the item's blocks: [w_begin, w_begin + nw)
  const int n_item_blk = blk_end - blk_begin;
  const int per_wave = (n_item_blk + kWavesPerGroup - 1) / kWavesPerGroup;
  const int w_begin = blk_begin + wave * per_wave;
  const int nw = __builtin_amdgcn_readfirstlane(max(0, min(per_wave, blk_end - w_begin)));
  // The block table is read-only for the whole launch: reading it through the constant
  // address space makes these uniform loads scalar (tracked apart from the vector loads).
  typedef const __attribute__((address_space(4))) int32_t* const_ids_t;
  const const_ids_t wave_ids = (const_ids_t)(reinterpret_cast<uintptr_t>(table + w_begin));

  __shared__ __attribute__((aligned(16))) uint16_t s_p[kWavesPerGroup][G][kBlockTokens];
  __shared__ float s_f[kWavesPerGroup][3][G];
  __shared__ float s_acc[kWavesPerGroup][G][D];

  u32x4 qreg[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const uint16_t* qp = a.q + (static_cast<int64_t>(b) * a.n_q_heads + h * G + g) * D + c * 8;
    qreg[g] = *reinterpret_cast<const u32x4*>(qp);
  }
  // Pin the query registers here: otherwise their loads are still counted as pending at
  // the head of the main loop and every iteration drains the whole load queue for them.
#pragma unroll
  for (int g = 0; g < G; ++g) asm volatile("" : "+v"(qreg[g]));

  float m_ref[VPL], l_exact[VPL], l_round[VPL], acc[G][NI];
#pragma unroll
  for (int v = 0; v < VPL; ++v) {
    m_ref[v] = -INFINITY;
    l_exact[v] = 0.0f;
    l_round[v] = 0.0f;
  }
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int i = 0; i < NI; ++i) acc[g][i] = 0.0f;

  // Physical block ids travel through the scalar cache, one ring entry per pipeline stage,
  // each fetched a full round (PF blocks) before the loads that need it are issued.
  int id_ring[PF];
#pragma unroll
  for (int s = 0; s < PF; ++s) id_ring[s] = nw > 0 ? wave_ids[min(s, nw - 1)] : 0;

  u32x4 kreg[PF][NI], vreg[PF][NI];
  const int64_t head_stride = 2 * kTileElems;
  const int64_t block_stride = static_cast<int64_t>(a.n_kv_heads) * head_stride;
  const int lane_elem_k = r * D + c * 8;           // K tile [16][D]
  const int lane_elem_v = kTileElems + lane * 8;   // V tile [D][16]: row lane/2 (+32 per load), tokens half*8..

  auto issue = [&](int stage, int j) {
    const int phys = id_ring[stage];
    id_ring[stage] = wave_ids[min(j + PF, nw - 1)];
    const uint16_t* tile = a.pool + static_cast<int64_t>(phys) * block_stride + h * head_stride;
#pragma unroll
    for (int i = 0; i < NI; ++i)
      kreg[stage][i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tile + i * TPI * D + lane_elem_k));
#pragma unroll
    for (int i = 0; i < NI; ++i)
      vreg[stage][i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tile + i * 512 + lane_elem_v));
  };

  auto compute = [&](int stage, int j) {
    const int n_valid = len - (w_begin + j) * kBlockTokens;   // >= 1; < 16 only in the last block

    // ---- logits: partial dots, then reduce-scatter over the lanes of each K row
    float part[N];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int g = 0; g < G; ++g) part[i * G + g] = dot8(qreg[g], kreg[stage][i], 0.0f);
    float z[VPL];
    row_reduce_scatter<LPR, N>(part, z, lane);
    const bool dead = my_tok >= n_valid;            // slots past the length may hold anything
#pragma unroll
    for (int v = 0; v < VPL; ++v) z[v] = dead ? -INFINITY : z[v] * a.scale_log2;

    // ---- lazily moved reference maximum
    bool grow = false;
#pragma unroll
    for (int v = 0; v < VPL; ++v) grow |= z[v] > m_ref[v] + kLazyMaxSlack;
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {
#pragma unroll
      for (int v = 0; v < VPL; ++v) {
        const float m_new = fmaxf(m_ref[v], same_head_max(z[v]));
        const float shrink = __builtin_amdgcn_exp2f(m_ref[v] - m_new);
        l_exact[v] *= shrink;
        l_round[v] *= shrink;
        m_ref[v] = m_new;
        if (lane < kSameHeadStride) s_f[wave][0][my_g0 + v] = shrink;
      }
      wave_lds_fence();
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float shrink = s_f[wave][0][g];
#pragma unroll
        for (int i = 0; i < NI; ++i) acc[g][i] *= shrink;
      }
    }

    // ---- p, rounded to bf16, to the wave's LDS row of its head
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      const float p = __builtin_amdgcn_exp2f(z[v] - m_ref[v]);
      const uint16_t pb = f32_to_bf16_rne(p);
      l_exact[v] += p;
      l_round[v] += __builtin_bit_cast(float, static_cast<uint32_t>(pb) << 16);
      s_p[wave][my_g0 + v][my_tok] = pb;
    }
    wave_lds_fence();

    // ---- V: 8 tokens of one head-dim element per lane and load
    if (n_valid < kBlockTokens) {                    // wave-uniform: zero the dead tokens' columns
      const int nv = n_valid - half * 8;
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        u32x4 vv = vreg[stage][i];
        vv.x &= (0 < nv ? 0x0000ffffu : 0u) | (1 < nv ? 0xffff0000u : 0u);
        vv.y &= (2 < nv ? 0x0000ffffu : 0u) | (3 < nv ? 0xffff0000u : 0u);
        vv.z &= (4 < nv ? 0x0000ffffu : 0u) | (5 < nv ? 0xffff0000u : 0u);
        vv.w &= (6 < nv ? 0x0000ffffu : 0u) | (7 < nv ? 0xffff0000u : 0u);
        vreg[stage][i] = vv;
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const u32x4 pp = *reinterpret_cast<const u32x4*>(&s_p[wave][g][half * 8]);
#pragma unroll
      for (int i = 0; i < NI; ++i) acc[g][i] = dot8(pp, vreg[stage][i], acc[g][i]);
    }
    wave_lds_fence();
  };

  // The steady-state loop is entered only behind an unconditional prologue: the compiler
  // places its load-queue waits from what may be pending on *any* path into the loop, and a
  // prologue with skipped stages would make it drain the queue in every iteration.
  int j = 0;
  if (nw >= 2 * PF) {
#pragma unroll
    for (int s = 0; s < PF; ++s) {
      issue(s, s);
      __builtin_amdgcn_sched_barrier(0);   // loads return in issue order: keep stage 0 first
    }
    for (; j + 2 * PF <= nw; j += PF) {
#pragma unroll
      for (int s = 0; s < PF; ++s) {
        compute(s, j + s);
        issue(s, j + s + PF);
      }
    }
  } else {
#pragma unroll
    for (int s = 0; s < PF; ++s)
      if (s < nw) issue(s, s);
  }
  for (; j < nw; j += PF) {               // drain: fewer than 2*PF blocks left
#pragma unroll
    for (int s = 0; s < PF; ++s) {
      if (j + s < nw) {
        compute(s, j + s);
        if (j + s + PF < nw) issue(s, j + s + PF);
      }
    }
  }

  // ---- wave totals: the two token halves of each head-dim element sit in lanes l, l ^ 1;
  //      the softmax sums of a head are spread over the lanes that carry that head
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int i = 0; i < NI; ++i) acc[g][i] = dpp_add<kDppXor1>(acc[g][i]);
#pragma unroll
  for (int v = 0; v < VPL; ++v) {
    l_exact[v] = same_head_sum(l_exact[v]);
    l_round[v] = same_head_sum(l_round[v]);
  }

  // ---- merge the four waves through LDS and store the item's partial result
  wave_lds_fence();
  if (half == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int i = 0; i < NI; ++i) s_acc[wave][g][i * 32 + (lane >> 1)] = acc[g][i];
  }
  if (lane < kSameHeadStride) {
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      s_f[wave][0][my_g0 + v] = m_ref[v];
      s_f[wave][1][my_g0 + v] = l_round[v];
      s_f[wave][2][my_g0 + v] = l_exact[v];
    }
  }
  __syncthreads();

  // Merged (reference max, sums, accumulator) of the four waves for output element (g, e).
  auto wave_merge = [&](int g, int e, float& M, float& val, float& Lr, float& Le) {
    M = s_f[0][0][g];
#pragma unroll
    for (int w = 1; w < kWavesPerGroup; ++w) M = fmaxf(M, s_f[w][0][g]);
    val = 0.0f, Lr = 0.0f, Le = 0.0f;
#pragma unroll
    for (int w = 0; w < kWavesPerGroup; ++w) {
      const float f = __builtin_amdgcn_exp2f(s_f[w][0][g] - M);   // 0 for a wave that had no block
      val = fmaf(f, s_acc[w][g][e], val);
      Lr = fmaf(f, s_f[w][1][g], Lr);
      Le = fmaf(f, s_f[w][2][g], Le);
    }
  };
  const int ns = rec.nsplit;
  const int64_t oj0 = static_cast<int64_t>(b) * a.n_q_heads + h * G;

  if (ns == 1) {                            // the item is the whole trajectory: finish it here
    for (int idx = threadIdx.x; idx < G * D; idx += kWavesPerGroup * 64) {
      const int g = idx / D, e = idx - g * D;
      float M, val, Lr, Le;
      wave_merge(g, e, M, val, Lr, Le);
      a.out[(oj0 + g) * D + e] = f32_to_bf16_rne(val / Lr);
      if (a.lse != nullptr && e == 0) a.lse[oj0 + g] = (M + __builtin_log2f(Le)) * 0.6931471805599453f;
    }
    return;
  }

  for (int idx = threadIdx.x; idx < G * D; idx += kWavesPerGroup * 64) {
    const int g = idx / D, e = idx - g * D;
    float M, val, Lr, Le;
    wave_merge(g, e, M, val, Lr, Le);
    const int64_t pj = static_cast<int64_t>(slot) * a.n_q_heads + h * G + g;
    a.part_acc[pj * D + e] = val;
    if (e == 0) {
      a.part_ml[pj * 4 + 0] = M;
      a.part_ml[pj * 4 + 1] = Lr;
      a.part_ml[pj * 4 + 2] = Le;
    }
  }
}

// Merges the parts of every trajectory that was split; one workgroup per (trajectory, query
// head).  (Merging inside the split-K kernel by the last item to arrive was tried: the
// device-scope fences it needs write back and invalidate the per-XCD L2 and doubled the
// kernel's duration.)
template <int D>
__global__ __launch_bounds__(D) void decode_combine_kernel(DecodeLaunch a) {
  const int b = blockIdx.x / a.n_q_heads;
  const DecodeTrajRec tr = a.trajs[b];
  const int ns = tr.nsplit;
  if (ns == 1) return;                      // finished by its only item
  const int j = blockIdx.x - b * a.n_q_heads;
  const int e = threadIdx.x;
  const int p0 = tr.part_off;
  // Parts are taken eight at a time, all loads of a round issued together (a part index past the
  // last one repeats the last part with weight 0), and merged into the running state with the
  // reference maximum moved as in the kernels; up to eight parts this is the plain two-pass form.
  float M = -INFINITY, num = 0.0f, den = 0.0f, den_exact = 0.0f;
  for (int s0 = 0; s0 < ns; s0 += 8) {
    float m[8], l[8], lx[8], ac[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int64_t pj = static_cast<int64_t>(p0 + min(s0 + i, ns - 1)) * a.n_q_heads + j;
      const float4 ml = *reinterpret_cast<const float4*>(a.part_ml + pj * 4);
      m[i] = s0 + i < ns ? ml.x : -INFINITY;
      l[i] = ml.y;
      lx[i] = ml.z;
      ac[i] = a.part_acc[pj * D + e];
    }
    float m_new = M;
#pragma unroll
    for (int i = 0; i < 8; ++i) m_new = fmaxf(m_new, m[i]);
    const float keep = __builtin_amdgcn_exp2f(M - m_new);     // 0 in the first round (nothing kept yet)
    num *= keep;
    den *= keep;
    den_exact *= keep;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float f = __builtin_amdgcn_exp2f(m[i] - m_new);
      den = fmaf(f, l[i], den);
      den_exact = fmaf(f, lx[i], den_exact);
      num = fmaf(f, ac[i], num);
    }
    M = m_new;
  }
  const int64_t oj = static_cast<int64_t>(a.out_row != nullptr ? a.out_row[b] : b) * a.n_q_heads + j;
  a.out[oj * D + e] = f32_to_bf16_rne(num / den);
  if (a.lse != nullptr && e == 0) a.lse[oj] = (M + __builtin_log2f(den_exact)) * 0.6931471805599453f;
}

template <int G, int D, int PF>
hipError_t launch_splitk(const DecodeLaunch& a, hipStream_t stream) {
  const dim3 grid(static_cast<unsigned>(a.n_items) * static_cast<unsigned>(a.n_kv_heads));
  hipLaunchKernelGGL((decode_splitk_kernel<G, D, PF>), grid, dim3(kWavesPerGroup * 64), 0, stream, a);
  return hipGetLastError();
}

}  // namespace

bool decode_shape_supported(int32_t group, int32_t head_dim) {
  return (head_dim == 64 || head_dim == 128) && (group == 1 || group == 2 || group == 4 || group == 8);
}

hipError_t launch_decode_splitk(const DecodeLaunch& a, hipStream_t stream) {
  const int G = a.n_q_heads / a.n_kv_heads;
  if (a.head_dim == 128) {
    switch (G) {
      case 1: return launch_splitk<1, 128, 3>(a, stream);
      case 2: return launch_splitk<2, 128, 3>(a, stream);
      case 4: return launch_splitk<4, 128, 3>(a, stream);
      case 8: return launch_splitk<8, 128, 3>(a, stream);
    }
  } else if (a.head_dim == 64) {
    switch (G) {
      case 1: return launch_splitk<1, 64, 3>(a, stream);
      case 2: return launch_splitk<2, 64, 3>(a, stream);
      case 4: return launch_splitk<4, 64, 3>(a, stream);
      case 8: return launch_splitk<8, 64, 3>(a, stream);
    }
  }
  return hipErrorInvalidValue;
}

hipError_t launch_decode_combine(const DecodeLaunch& a, hipStream_t stream) {
  const dim3 grid(static_cast<unsigned>(a.B) * static_cast<unsigned>(a.n_q_heads));
  if (a.head_dim == 128)
    hipLaunchKernelGGL((decode_combine_kernel<128>), grid, dim3(128), 0, stream, a);
  else
    hipLaunchKernelGGL((decode_combine_kernel<64>), grid, dim3(64), 0, stream, a);
  return hipGetLastError();
}

}  // namespace heddle
