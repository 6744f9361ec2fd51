// Prefill attention (Section 3.2, prefill phase: the prompt's own attention is computed on the
// full-precision K and V before anything is quantized; Algorithm 1 with h = 0, l = len(prompt))
// for gfx950: causal softmax attention of fp16 Q, K, V with fp32 accumulation, one pass over the
// keys with a running maximum and sum per query (online softmax).
//
// One workgroup of 8 wavefronts owns 256 consecutive queries of one (sequence, query head); a
// wavefront owns 32 of them (every tile of K and V that the workgroup fetches serves 256 queries:
// at 128 the kernel was bound by the K/V traffic from L2 and HBM).  Keys and values arrive in
// tiles of 64 tokens, staged in LDS (K as it is, V transposed so that the keys of one channel are
// neighbours, in an order that lets a lane fetch each operand of the value product with one
// 16-byte read and spreads the transposing stores over the banks), double buffered: while a tile
// is computed the next one travels from HBM into registers.  Per wavefront and tile:
//   S^T[key][query]  by 16 v_mfma_f32_32x32x16_f16: A = K tile (row = key, 16 channels a step),
//        B = the wavefront's queries, held in registers for the whole kernel.  Computing the
//        transpose puts the 32 scores that a lane holds (of 64) in the column of ONE query, so the
//        running maximum and sum need one cross-lane exchange, and
//   O^T[channel][query]  by 32 more: A = V^T tile, B = P^T, which is exactly what the lane
//        already holds: its exp2'd scores, converted to fp16, are the B operand as they are (the
//        order of the keys inside a step of 16 is the accumulator's: both operands use it).  Every
//        weight enters twice, as a high and a low fp16 part on the same A operand, so that the
//        output keeps ~22 bits of the weights (one fp16 part alone: an error up to 2^-12 max|V|).
// Causality: a workgroup stops at the last tile its queries can see, a wavefront skips the tiles
// beyond its own queries, and only tiles that straddle the diagonal are masked element-wise.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <math.h>

#include "skvq_internal.h"

namespace skvq {
namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef unsigned uint2_t __attribute__((ext_vector_type(2)));
typedef unsigned uint4_t __attribute__((ext_vector_type(4)));

constexpr int kQBlock = 256;    // queries per workgroup (32 per wavefront)
constexpr int kThreads = 2 * kQBlock;
constexpr int kKTile = 64;      // keys per tile
constexpr int kKStride = 136;   // halves per K row in LDS (272 B: 16-byte aligned, rows on different banks)
constexpr int kVStride = 72;    // halves per V^T row in LDS (144 B: 16-byte aligned, rows on different banks)
constexpr float kLog2e = 1.4426950408889634f;
// The running reference sits kBias below the largest score it was set from (that key's weight is
// 2^kBias) and moves when a score exceeds it by more than kSlack: weights stay below 2^15, which fp16
// holds, and a weight only falls under fp16's smallest step (2^-24) when it is 2^-31 of the largest.
constexpr float kBias = 7.0f, kSlack = 15.0f;

// max(a, b, c) in one instruction (the plain fmaxf first re-canonicalizes every matrix-core result)
__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

struct Smem {
  _Float16 k[2][kKTile][kKStride];  // [buffer][key][channel]
  _Float16 vt[2][kD][kVStride];     // [buffer][channel][key, in the order that store_v describes]
};

// What one thread carries of a tile between HBM and LDS: 2 pieces of 8 channels of K (keys
// tid/16 + 32 i) and a 2-key x 8-channel block of V (keys 2 (tid/16), 2 (tid/16) + 1).
struct Stage {
  uint4_t k[2], v[2];
};

__global__ __launch_bounds__(kThreads, 2) void prefill_attn_kernel(const __half *__restrict__ q,
                                                              const __half *__restrict__ k,
                                                              const __half *__restrict__ v, float *__restrict__ out_f32,
                                                              __half *__restrict__ out_f16, int T, int Hq, int Hk,
                                                              float sm_scale) {
  __shared__ __align__(16) Smem sm;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, h = lane >> 5;
  const int n_qblocks = (T + kQBlock - 1) / kQBlock;
  const int qb = n_qblocks - 1 - (int)blockIdx.x;  // the longest blocks start first
  const int hq = blockIdx.y, b = blockIdx.z, hk = hq / (Hq / Hk);
  const __half *qh = q + ((size_t)b * Hq + hq) * (size_t)T * kD;
  const __half *kh = k + ((size_t)b * Hk + hk) * (size_t)T * kD;
  const __half *vh = v + ((size_t)b * Hk + hk) * (size_t)T * kD;
  const float c = sm_scale * kLog2e;

  const int q0 = qb * kQBlock + 32 * wave;           // this wavefront's first query
  const int my_q = q0 + col;                         // this lane's query (two lanes share one)
  const int last_q_block = min(qb * kQBlock + kQBlock - 1, T - 1);
  const int n_tiles = last_q_block / kKTile + 1;     // tiles the workgroup's queries can see
  const int wave_last_q = min(q0 + 31, T - 1);       // (q0 may lie beyond T: then nothing is stored)
  const int wave_tiles = q0 < T ? wave_last_q / kKTile + 1 : 0;

  // the queries: B operand of the score product, channels 16 s + 8 h .. + 7 for step s
  uint4_t qreg[8];
  {
    const int qrow = min(my_q, T - 1);
    const uint4_t *src = reinterpret_cast<const uint4_t *>(qh + (size_t)qrow * kD);
#pragma unroll
    for (int s = 0; s < 8; ++s) qreg[s] = src[2 * s + h];
  }

  auto load_k = [&](Stage &st, int tile) {
    const int kq = tid >> 4, dc = tid & 15;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int key = min(tile * kKTile + kq + 32 * i, T - 1);  // rows past the end repeat the last one (masked)
      st.k[i] = reinterpret_cast<const uint4_t *>(kh + (size_t)key * kD)[dc];
    }
  };
  auto load_v = [&](Stage &st, int tile) {
    const int kq = tid >> 4, dc = tid & 15;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int key = min(tile * kKTile + 2 * kq + r, T - 1);
      st.v[r] = reinterpret_cast<const uint4_t *>(vh + (size_t)key * kD)[dc];
    }
  };
  auto load_stage = [&](int tile) {
    Stage st;
    load_k(st, tile);
    load_v(st, tile);
    return st;
  };
  auto store_k = [&](const Stage &st, int buf) {
    const int kq = tid >> 4, dc = tid & 15;
#pragma unroll
    for (int i = 0; i < 2; ++i) *reinterpret_cast<uint4_t *>(&sm.k[buf][kq + 32 * i][8 * dc]) = st.k[i];
  };
  auto store_v = [&](const Stage &st, int buf) {
    const int kq = tid >> 4, dc = tid & 15;
    // Inside a row the 64 keys sit in eight 16-byte cells: cell 2 (key / 16) + (key / 4) % 2 holds
    // keys 16 g + 4 h + {0..3} and 16 g + 8 + 4 h + {0..3}, the eight that one lane feeds to a step
    // of the value product, and the cells of a row are permuted by the row's channel block
    // (cell ^ 2 blk), which spreads the transposing stores of a wavefront over the banks
    const int kcol = 8 * ((2 * (kq >> 3) + ((kq >> 1) & 1)) ^ (2 * (dc >> 2))) + 4 * ((kq >> 2) & 1) + 2 * (kq & 1);
    // transpose the 2 x 8 block: channel 8 dc + d gets its two keys as one dword
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const unsigned a0 = st.v[0][j], a1 = st.v[1][j];
      *reinterpret_cast<unsigned *>(&sm.vt[buf][8 * dc + 2 * j][kcol]) = __builtin_amdgcn_perm(a1, a0, 0x05040100u);
      *reinterpret_cast<unsigned *>(&sm.vt[buf][8 * dc + 2 * j + 1][kcol]) = __builtin_amdgcn_perm(a1, a0, 0x07060302u);
    }
  };

  // (-1 as a value the compiler cannot see through: p - hi then stays one mixed-precision
  // multiply-add on the fp16 operand instead of a conversion and a subtraction)
  float minus_one = -1.0f;
  asm("" : "+v"(minus_one));
  float16_t o[4];  // O^T: channel 32 blk + 8 (x/4) + 4 h + x%4 of this lane's query
#pragma unroll
  for (int blk = 0; blk < 4; ++blk)
#pragma unroll
    for (int x = 0; x < 16; ++x) o[blk][x] = 0.f;
  float m = -INFINITY, l = 0.f;  // running maximum (log2 domain) and this lane's part of the sum

  // Scores of tile `tile` from K buffer `kbuf`: sixteen products, two alternating accumulation
  // chains (key blocks), the LDS operand reads kept four ahead of the products.
  auto scores = [&](int kbuf, float16_t (&s)[2]) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int x = 0; x < 16; ++x) s[kb][x] = 0.f;
    half8_t a[2][4];  // [parity of the batch][2 * (ds % 2) + kb]
    auto read_batch = [&](int bt) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int ds = 2 * bt + (i >> 1), kb = i & 1;
        a[bt & 1][i] = *reinterpret_cast<const half8_t *>(&sm.k[kbuf][32 * kb + col][16 * ds + 8 * h]);
      }
    };
    read_batch(0);
#pragma unroll
    for (int bt = 0; bt < 4; ++bt) {
      if (bt + 1 < 4) read_batch(bt + 1);
      __builtin_amdgcn_sched_barrier(0);  // keep the reads ahead of the products
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int ds = 2 * bt + (i >> 1), kb = i & 1;
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[bt & 1][i], __builtin_bit_cast(half8_t, qreg[ds]), s[kb], 0, 0, 0);
      }
    }
  };

  // The K tiles run one tile ahead of the V tiles: while a wavefront turns the scores of tile j
  // into weights on the vector ALU, the matrix core already works on the scores of tile j + 1.
  float16_t s_a[2], s_b[2];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int x = 0; x < 16; ++x) s_a[kb][x] = s_b[kb][x] = 0.f;
  {
    Stage st0 = load_stage(0), st1 = load_stage(min(1, n_tiles - 1));
    store_k(st0, 0);
    store_v(st0, 0);
    store_k(st1, 1);
  }
  __syncthreads();
  // Every load issued so far must have landed before the loop: the compiler counts the loads in
  // flight at the loop's top over all paths into it, and a query load still pending on entry
  // would turn into a wait for the NEXT tile's loads on every later trip.
  asm volatile("" ::"v"(qreg[0]), "v"(qreg[1]), "v"(qreg[2]), "v"(qreg[3]), "v"(qreg[4]), "v"(qreg[5]), "v"(qreg[6]),
               "v"(qreg[7]));
  if (0 < wave_tiles) scores(0, s_a);
  __syncthreads();  // K buffer 0 is overwritten at the end of the first trip

  // One trip: the scores of tile + 1 into s_next, softmax and value product of tile from s_cur.
  // The loop below runs trips in pairs with the two score buffers swapping roles (no register
  // copies); an odd tile count gets one idle trip (its loads repeat the last tile, its products
  // are skipped, its stores go to buffers that nobody reads any more).
  auto trip = [&](const int tile, float16_t (&s_cur)[2], float16_t (&s_next)[2]) {
    const int buf = tile & 1;
    // K of tile + 2 and V of tile + 1, in flight during the products below (unconditional: past
    // the last tile the last one is fetched and stored again, which nobody reads)
    Stage st;
    load_k(st, min(tile + 2, n_tiles - 1));
    load_v(st, min(tile + 1, n_tiles - 1));

    if (tile + 1 < wave_tiles) scores(buf ^ 1, s_next);  // runs on the matrix core during the softmax below

    if (tile < wave_tiles) {
      float16_t(&s)[2] = s_cur;
      // key of s[kb][x]: tile*64 + 32 kb + 8 (x/4) + 4 h + x%4
      if (tile * kKTile + kKTile - 1 > q0) {  // some key of the tile lies beyond some query: mask
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int x = 0; x < 16; ++x) {
            const int key = tile * kKTile + 32 * kb + 8 * (x >> 2) + 4 * h + (x & 3);
            if (key > my_q) s[kb][x] = -INFINITY;
          }
      }
      // The running reference m only moves when a score exceeds it by more than kSlack (log2
      // domain): the weights stay below 2^kSlack, and the accumulators are rescaled on few
      // tiles.  (Key 0 is visible to every query, so the first tile sets a finite reference.)
      float mloc = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int x = 0; x < 16; x += 2) mloc = max3(mloc, s[kb][x], s[kb][x + 1]);
      {  // the other half of the query's scores is 32 lanes away: one swap of register halves
        // (lanes 32-63 of the first register trade places with lanes 0-31 of the second)
        float ma = mloc, mb = mloc;
        asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(ma), "+v"(mb));
        mloc = max3(ma, mb, mb) * c;  // c >= 0
      }
      if (__any(mloc > m + kSlack)) {
        const float m_new = fmaxf(m, mloc - kBias);
        const float alpha = exp2f(m - m_new);  // 0 at the first tile
        m = m_new;
        l *= alpha;
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
#pragma unroll
          for (int x = 0; x < 16; ++x) o[blk][x] *= alpha;
      }
      float psum = 0.f;
      // B operands of the value product: step t covers keys 16 t .. 16 t + 15 of the tile.  A weight
      // enters as two fp16 numbers, its top 11 significant bits (converted toward zero; the
      // difference to the fp32 value is exact and comes from one mixed-precision multiply-add) and
      // the rest (rounded toward zero to 11 more): ~22 bits in all, so the
      // weights' rounding stays below 2^-21 of the largest value instead of 2^-12.
      uint4_t p[4], plo[4];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int x = 0; x < 16; x += 2) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(s[kb][x], c, -m));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(s[kb][x + 1], c, -m));
          psum += p0 + p1;
          const auto hi = __builtin_amdgcn_cvt_pkrtz(p0, p1);  // toward zero: the top 11 significant bits
          const float l0 = __builtin_fmaf((float)hi[0], minus_one, p0), l1 = __builtin_fmaf((float)hi[1], minus_one, p1);  // exact
          p[2 * kb + (x >> 3)][(x & 7) >> 1] = __builtin_bit_cast(unsigned, hi);
          plo[2 * kb + (x >> 3)][(x & 7) >> 1] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(l0, l1));
        }
      l += psum;
      // ---- values: the lane's slot e of step t is key 16 t + 8 (e/4) + 4 h + e%4 ----
      auto v_operand = [&](int t, int blk) {
        return *reinterpret_cast<const half8_t *>(&sm.vt[buf][32 * blk + col][16 * (t ^ blk) + 8 * h]);
      };
      half8_t va[2][2];  // the A operands of half a step (two channel blocks), requested half a step ahead
#pragma unroll
      for (int i = 0; i < 2; ++i) va[0][i] = v_operand(0, i);
#pragma unroll
      for (int hs = 0; hs < 8; ++hs) {  // half step: step hs / 2, channel blocks 2 (hs % 2), + 1
        if (hs + 1 < 8) {
#pragma unroll
          for (int i = 0; i < 2; ++i) va[(hs + 1) & 1][i] = v_operand((hs + 1) >> 1, 2 * ((hs + 1) & 1) + i);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          const int blk = 2 * (hs & 1) + i;
          o[blk] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va[hs & 1][i], __builtin_bit_cast(half8_t, p[hs >> 1]), o[blk], 0, 0, 0);
          o[blk] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va[hs & 1][i], __builtin_bit_cast(half8_t, plo[hs >> 1]), o[blk], 0, 0, 0);
        }
      }
    }
    // K of tile + 2 replaces K of tile (read during the previous trip), V of tile + 1 replaces V
    // of tile - 1: nobody reads either buffer during this trip
    store_k(st, buf);
    store_v(st, buf ^ 1);
    __syncthreads();
  };
  for (int tile = 0; tile < n_tiles; tile += 2) {
    trip(tile, s_a, s_b);
    trip(tile + 1, s_b, s_a);
  }

  // ---- epilogue: divide by the sum, store channel-contiguous pieces of 4 ----
  const float lt = l + __shfl_xor(l, 32);
  if (my_q < T) {
    const float inv = 1.f / lt;
    const size_t row = (((size_t)b * Hq + hq) * (size_t)T + my_q) * kD;
#pragma unroll
    for (int blk = 0; blk < 4; ++blk)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int ch = 32 * blk + 8 * g + 4 * h;
        const float4_t val = {o[blk][4 * g] * inv, o[blk][4 * g + 1] * inv, o[blk][4 * g + 2] * inv,
                              o[blk][4 * g + 3] * inv};
        *reinterpret_cast<float4_t *>(out_f32 + row + ch) = val;
        if (out_f16) {
          const __half2 lo2 = __floats2half2_rn(val[0], val[1]), hi2 = __floats2half2_rn(val[2], val[3]);
          *reinterpret_cast<uint2_t *>(out_f16 + row + ch) =
              uint2_t{__builtin_bit_cast(unsigned, lo2), __builtin_bit_cast(unsigned, hi2)};
        }
      }
  }
}

}  // namespace

hipError_t launch_prefill_attention(const Layout &L, const __half *q, const __half *k, const __half *v,
                                    float *out_f32, __half *out_f16, long long T, hipStream_t s) {
  if (T <= 0 || T > 0x3fffffffll || L.Hq > 65535 || L.B > 65535) return hipErrorInvalidValue;
  const int n_qblocks = (int)((T + kQBlock - 1) / kQBlock);
  hipLaunchKernelGGL(prefill_attn_kernel, dim3(n_qblocks, L.Hq, L.B), dim3(kThreads), 0, s, q, k, v, out_f32, out_f16,
                     (int)T, L.Hq, L.Hk, L.sm_scale);
  return hipGetLastError();
}

}  // namespace skvq
