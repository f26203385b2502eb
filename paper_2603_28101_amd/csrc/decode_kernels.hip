// Split-K decode attention over a paged KV pool, and the log-sum-exp merge of its parts.
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
// Lane layout (wave64): a K or V row of d bf16 is covered by d/8 lanes holding 8 elements
// (16 bytes) each, so one wave load instruction brings 64*16 B = 1 KB = 1024/(2d) token
// rows.  Each lane forms G partial dot products with packed-bf16 dot instructions, the
// d/8 lanes of a row are summed with DPP adds, and the same lane layout is reused for
// V, so P*V needs no data movement: acc[g][8] += p[g] * v[8].
//
// Softmax runs in base 2 with a lazily updated reference maximum per head: the reference
// only moves (and the accumulators are only rescaled) when some logit exceeds it by more
// than 2^8, which is rare after the first few blocks; p is then at most 256.
#include "kernels.h"

namespace heddle {

namespace {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kBlockTokens = 16;
constexpr int kWavesPerGroup = 4;
constexpr float kLazyMaxSlack = 8.0f;   // log2 units

template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true);
  return x + __builtin_bit_cast(float, moved);
}

// Sum over the LPR consecutive lanes that hold one token row; every lane gets the sum.
// N independent values go through each step together so that the two wait states a DPP
// read needs after a VALU write are filled by the neighbouring chains.
template <int LPR, int N>
__device__ __forceinline__ void row_sum(float (&x)[N]) {
  if constexpr (LPR == 16) {
#pragma unroll
    for (int n = 0; n < N; ++n) x[n] = dpp_add<0x128>(x[n]);   // row_ror:8
  }
#pragma unroll
  for (int n = 0; n < N; ++n) x[n] = dpp_add<0x141>(x[n]);     // row_half_mirror
#pragma unroll
  for (int n = 0; n < N; ++n) x[n] = dpp_add<0xB1>(x[n]);      // quad_perm [1,0,3,2]
#pragma unroll
  for (int n = 0; n < N; ++n) x[n] = dpp_add<0x4E>(x[n]);      // quad_perm [2,3,0,1]
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x = fmaxf(x, __shfl_xor(x, off, 64));
  return x;
}

// The packed operands go through a by-value helper: a bit cast applied directly to a
// vector element (v.y) reads element 0 with this compiler.
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}

__device__ __forceinline__ float dot8(const u32x4& a, const u32x4& b) {
  float s = dot2(a.x, b.x, 0.0f);
  s = dot2(a.y, b.y, s);
  s = dot2(a.z, b.z, s);
  s = dot2(a.w, b.w, s);
  return s;
}

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __builtin_bit_cast(float, u & 0xffff0000u); }

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

// G: query heads per kv head.  D: head dim.  PF: KV blocks kept in flight per wave.
template <int G, int D, int PF>
__global__ __launch_bounds__(kWavesPerGroup * 64, 2) void decode_splitk_kernel(DecodeLaunch a) {
  constexpr int LPR = D / 8;          // lanes per token row
  constexpr int TPI = 64 / LPR;       // token rows per wave load instruction
  constexpr int NI = kBlockTokens / TPI;  // load instructions per K (or V) tile of one block
  constexpr int kTileElems = kBlockTokens * D;

  const int item = blockIdx.x / a.n_kv_heads;
  const int h = blockIdx.x - item * a.n_kv_heads;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = lane / LPR;           // token row within a load instruction
  const int c = lane - r * LPR;       // 8-element slice of the head dim

  const int b = a.item_b[item];
  const int blk_begin = a.item_blk_begin[item];
  const int blk_end = a.item_blk_end[item];
  const int len = a.lens[b];
  const int32_t* table = a.block_ids + a.row_off[b];
  const int slot = a.part_off[b] + a.item_s[item];

  // each wave streams a contiguous quarter of the item's blocks: [w_begin, w_begin + nw)
  const int n_item_blk = blk_end - blk_begin;
  const int per_wave = (n_item_blk + kWavesPerGroup - 1) / kWavesPerGroup;
  const int w_begin = blk_begin + wave * per_wave;
  const int nw = __builtin_amdgcn_readfirstlane(max(0, min(per_wave, blk_end - w_begin)));
  // The block table is read-only for the whole launch: reading it through the constant
  // address space makes these uniform loads scalar (tracked apart from the vector loads).
  typedef const __attribute__((address_space(4))) int32_t* const_ids_t;
  const const_ids_t wave_ids = (const_ids_t)(reinterpret_cast<uintptr_t>(table + w_begin));

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

  float m_ref[G], l_sum[G], acc[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m_ref[g] = -INFINITY;
    l_sum[g] = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[g][e] = 0.0f;
  }

  // Physical block ids travel through the scalar cache, one ring entry per pipeline stage,
  // each fetched a full round (PF blocks) before the loads that need it are issued.
  int id_ring[PF];
#pragma unroll
  for (int s = 0; s < PF; ++s) id_ring[s] = nw > 0 ? wave_ids[min(s, nw - 1)] : 0;

  u32x4 kreg[PF][NI], vreg[PF][NI];
  const int64_t head_stride = 2 * kTileElems;
  const int64_t block_stride = static_cast<int64_t>(a.n_kv_heads) * head_stride;
  const int lane_elem_k = r * D + c * 8;
  const int lane_elem_v = lane_elem_k + kTileElems;

  auto issue = [&](int stage, int j) {
    const int phys = id_ring[stage];
    id_ring[stage] = wave_ids[min(j + PF, nw - 1)];
    const uint16_t* tile = a.pool + static_cast<int64_t>(phys) * block_stride + h * head_stride;
#pragma unroll
    for (int i = 0; i < NI; ++i)
      kreg[stage][i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tile + i * TPI * D + lane_elem_k));
#pragma unroll
    for (int i = 0; i < NI; ++i)
      vreg[stage][i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tile + i * TPI * D + lane_elem_v));
  };

  auto compute = [&](int stage, int j) {
    const int tok0 = (w_begin + j) * kBlockTokens;
    const int n_valid = len - tok0;                  // >= 1; < 16 only in a trajectory's last block
    float z[G][NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      float part[G];
#pragma unroll
      for (int g = 0; g < G; ++g) part[g] = dot8(qreg[g], kreg[stage][i]);
      row_sum<LPR, G>(part);
#pragma unroll
      for (int g = 0; g < G; ++g) z[g][i] = part[g] * a.scale_log2;
    }

    if (n_valid < kBlockTokens) {                    // wave-uniform: ragged tail of the context
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const bool dead = i * TPI + r >= n_valid;
        if (dead) {
          vreg[stage][i] = u32x4{0u, 0u, 0u, 0u};     // slots past the length may hold NaN
#pragma unroll
          for (int g = 0; g < G; ++g) z[g][i] = -INFINITY;
        }
      }
    }

    bool grow = false;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float zmax = z[g][0];
#pragma unroll
      for (int i = 1; i < NI; ++i) zmax = fmaxf(zmax, z[g][i]);
      grow |= zmax > m_ref[g] + kLazyMaxSlack;
    }
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {    // rare: move the reference maximum
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float zmax = z[g][0];
#pragma unroll
        for (int i = 1; i < NI; ++i) zmax = fmaxf(zmax, z[g][i]);
        const float m_new = fmaxf(m_ref[g], wave_max(zmax));
        const float shrink = __builtin_amdgcn_exp2f(m_ref[g] - m_new);
        l_sum[g] *= shrink;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] *= shrink;
        m_ref[g] = m_new;
      }
    }

#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const u32x4 vv = vreg[stage][i];
      const float v[8] = {bf16_lo(vv.x), bf16_hi(vv.x), bf16_lo(vv.y), bf16_hi(vv.y),
                          bf16_lo(vv.z), bf16_hi(vv.z), bf16_lo(vv.w), bf16_hi(vv.w)};
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float p = __builtin_amdgcn_exp2f(z[g][i] - m_ref[g]);
        l_sum[g] += p;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = fmaf(p, v[e], acc[g][e]);
      }
    }
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

  // ---- merge the TPI token rows of the wave (lanes with equal c) ----
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      l_sum[g] += __shfl_xor(l_sum[g], off, 64);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[g][e] += __shfl_xor(acc[g][e], off, 64);
    }
  }

  // ---- merge the four waves through LDS and store the item's partial result ----
  __shared__ float s_acc[kWavesPerGroup][G][D];
  __shared__ float s_m[kWavesPerGroup][G];
  __shared__ float s_l[kWavesPerGroup][G];
  if (r == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int e = 0; e < 8; ++e) s_acc[wave][g][c * 8 + e] = acc[g][e];
      if (c == 0) {
        s_m[wave][g] = m_ref[g];
        s_l[wave][g] = l_sum[g];     // each row lane holds the same sum; rows were added above
      }
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < G * D; idx += kWavesPerGroup * 64) {
    const int g = idx / D;
    const int e = idx - g * D;
    float M = s_m[0][g];
#pragma unroll
    for (int w = 1; w < kWavesPerGroup; ++w) M = fmaxf(M, s_m[w][g]);
    float val = 0.0f, L = 0.0f;
#pragma unroll
    for (int w = 0; w < kWavesPerGroup; ++w) {
      const float f = __builtin_amdgcn_exp2f(s_m[w][g] - M);   // 0 for a wave that had no block
      val = fmaf(f, s_acc[w][g][e], val);
      L = fmaf(f, s_l[w][g], L);
    }
    const int64_t pj = static_cast<int64_t>(slot) * a.n_q_heads + h * G + g;
    a.part_acc[pj * D + e] = val;
    if (e == 0) {
      a.part_ml[pj * 2 + 0] = M;
      a.part_ml[pj * 2 + 1] = L;
    }
  }
}

// One workgroup per (trajectory, query head): merges the trajectory's parts.
template <int D>
__global__ __launch_bounds__(D) void decode_combine_kernel(DecodeLaunch a) {
  const int b = blockIdx.x / a.n_q_heads;
  const int j = blockIdx.x - b * a.n_q_heads;
  const int e = threadIdx.x;
  const int p0 = a.part_off[b];
  const int ns = a.nsplit[b];
  float M = -INFINITY;
  for (int s = 0; s < ns; ++s) M = fmaxf(M, a.part_ml[(static_cast<int64_t>(p0 + s) * a.n_q_heads + j) * 2]);
  float num = 0.0f, den = 0.0f;
  for (int s = 0; s < ns; ++s) {
    const int64_t pj = static_cast<int64_t>(p0 + s) * a.n_q_heads + j;
    const float f = __builtin_amdgcn_exp2f(a.part_ml[pj * 2] - M);
    den = fmaf(f, a.part_ml[pj * 2 + 1], den);
    num = fmaf(f, a.part_acc[pj * D + e], num);
  }
  const int64_t oj = static_cast<int64_t>(b) * a.n_q_heads + j;
  a.out[oj * D + e] = f32_to_bf16_rne(num / den);
  if (a.lse != nullptr && e == 0) a.lse[oj] = (M + __builtin_log2f(den)) * 0.6931471805599453f;
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
      case 8: return launch_splitk<8, 128, 2>(a, stream);
    }
  } else if (a.head_dim == 64) {
    switch (G) {
      case 1: return launch_splitk<1, 64, 3>(a, stream);
      case 2: return launch_splitk<2, 64, 3>(a, stream);
      case 4: return launch_splitk<4, 64, 3>(a, stream);
      case 8: return launch_splitk<8, 64, 2>(a, stream);
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
