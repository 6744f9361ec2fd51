// Matrix-core chunk kernel of skvq_decode_attention for gfx950 (group size 128, up to four
// query heads per kv head).
//
// Per wavefront, per tile of 64 packed tokens (lane = token for the score half):
//   QK   S^T[(token group, head)][token] by 16 v_mfma_f32_16x16x32_f16, four per group of 16
//        tokens: the B operand is 8 bytes of a key row (lane = (token, quarter of the row)),
//        its 2-bit codes turned into fp16 SUBNORMALS by one AND each (code c at mantissa bit
//        s is the fp16 value c*2^(s-24)); the A operand is the reordered query, pre-multiplied
//        by the matching power of two and placed in the rows of its token group (zero in the
//        other rows), held in registers.  All four groups accumulate into ONE 16x16 tile, so
//        afterwards lane l holds the scores of token l for the (up to) four heads.  Few, wide
//        products on purpose: the matrix core truncates when it accumulates, a few ulp per
//        instruction.
//   softmax  lazily re-referenced online softmax in the exp2 domain: the running reference
//        m only moves when a score exceeds it by more than 2^6 (wave-uniform branch).
//   PV   O^T[channel][head] by 16 v_mfma_f32_16x16x32_f16: the A operand is the V block unit
//        that the lane loaded (8 tokens x 8 channels, token-minor, again one AND per
//        register; 3-level units go through a 13-bit -> 8-code table in LDS), the B operand
//        holds p*scale split into a high and a low fp16 part (two columns per head) so that
//        the weights keep ~22 bits.
// The zero-points never enter the matrix products: sum_p q_p (s c_p + z) = s sum q c + z sum q
// and sum_t w_t (s_t c + z_t) = sum (w_t s_t) c + sum w_t z_t.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <math.h>

#include "skvq_internal.h"

namespace skvq {
namespace {

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef unsigned uint2_t __attribute__((ext_vector_type(2)));
typedef unsigned uint4_t __attribute__((ext_vector_type(4)));
struct __attribute__((aligned(4))) Unit16 {  // a 16-byte load that is only 4-byte aligned
  unsigned x, y, z, w;
};

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kRefSlack = 6.0f;       // scores may exceed the running reference by 2^6
constexpr float kVsTarget = 256.0f;     // max(v scale)*beta is brought below this ...
constexpr float kVsLimit = 512.0f;      // ... and re-normalised when a token exceeds this

__device__ __forceinline__ float wave_max(float v) {
  for (int off = 32; off; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  for (int off = 32; off; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// The 2-bit codes reach the matrix core as fp16 SUBNORMALS: a code c sitting at mantissa bit s
// is the value c*2^(s-24).  The core accumulates such products as if their mantissa were full,
// so a code at a low bit costs about (10 - s) bits of the accumulator's precision; every
// code is therefore moved to bit 4, 6 or 8 before it is masked out.
constexpr unsigned kM4 = 0x00300030u, kM6 = 0x00c000c0u, kM8 = 0x03000300u;

// Key dword (16 codes, position e at bit 2e) -> two B operands of the 16x16x32 product.
// Operand 0 holds positions e = {0,8,1,9,2,10,3,11} at bits s = {4,4,6,6,4,4,6,6};
// operand 1 holds e = {4,12,5,13,6,14,7,15} at s = {8,8,4,4,6,6,8,8}.
__device__ __forceinline__ void unpack_k(unsigned w, half8_t b[2]) {
  const unsigned wl = w << 4, wr = w >> 6;
  b[0] = __builtin_bit_cast(half8_t, uint4_t{wl & kM4, wl & kM6, w & kM4, w & kM6});
  b[1] = __builtin_bit_cast(half8_t, uint4_t{w & kM8, wr & kM4, wr & kM6, wr & kM8});
}

// For reordered position p: which quarter of the row (lane group kb), which of the quarter's
// four products, which k slot of that product, and the power of two the key code carries there.
__device__ __forceinline__ void k_slot_of(int p, int &kb, int &step, int &kslot, int &shift) {
  const int d = (p >> 4) & 1, e = p & 15, lo = e & 7, hi = e >> 3;  // e = lo + 8*hi
  kb = p >> 5;
  step = 2 * d + (lo >> 2);
  kslot = 2 * (lo & 3) + hi;
  const int tab = 0x86486464;          // bit position of code lo (and lo+8), one nibble each
  shift = (tab >> (4 * lo)) & 15;
}

// Eight tokens of one channel -> A operand of the 16x16x32 product: register m holds tokens
// 2m (low half) and 2m+1 (high half) at mantissa bit {4, 6, 8, 8}[m].
// From a table entry (pairs 0,1,2 at bits 4,6,8; pair 3 at bit 0):
__device__ __forceinline__ half8_t unpack_v_entry(unsigned e) {
  return __builtin_bit_cast(half8_t, uint4_t{e & kM4, e & kM6, e & kM8, (e << 8) & kM8});
}
// From a 2-bit unit field (pair m at bit 2m of each half; `f` has the field in bits 0..7):
__device__ __forceinline__ half8_t unpack_v_field(unsigned f) {
  const unsigned a = f << 4, b = f << 2;
  return __builtin_bit_cast(half8_t, uint4_t{a & kM4, a & kM6, a & kM8, b & kM8});
}

template <int R, bool TERNARY>
struct Smem {
  unsigned lut[TERNARY ? 8192 : 1];
  _Float16 qa[4][4][4][8];      // A operands of the score product: [row quarter][step][head][k slot]
  float qsum[4];                // sm_scale*log2(e) * sum of the query, per head
  float qinit[4];               // -1.5 * sum of the query, in the score product's units (2^-16)
  _Float16 pbuf[4][2][2 * R][32];  // per wave: [block][column][token slot]
  float stage[4][2 * R][kD];    // epilogue: O^T per wave and column
  float wm[4][R], wl[4][R], wz[4][R];
};

template <int R, bool TERNARY>
__global__ __launch_bounds__(256, 2) void decode_mfma_kernel(Layout L, const __half *__restrict__ q,
                                                             long long nq, long long tiles_per_split) {
  __shared__ Smem<R, TERNARY> sm;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sp = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
  const long long head = (long long)b * L.Hk + hk;
  const float c = L.sm_scale * kLog2e;

  // ---- prologue: table, query operands ----
  if (TERNARY) {
    const uint4_t *src = reinterpret_cast<const uint4_t *>(L.trit_lut);
    uint4_t *dst = reinterpret_cast<uint4_t *>(sm.lut);
    for (int x = tid; x < 2048; x += 256) dst[x] = src[x];
  }
  for (int x = tid; x < 4 * kD; x += 256) {
    const int r = x >> 7, p = x & 127;
    int kb, step, kslot, shift;
    k_slot_of(p, kb, step, kslot, shift);
    float v = 0.f;
    if (r < R) v = __half2float(q[((long long)b * L.Hq + hk * R + r) * kD + L.perm_k[hk * kD + p]]);
    sm.qa[kb][step][r][kslot] = (_Float16)ldexpf(v, 8 - shift);  // exact: a power of two
  }
  __syncthreads();
  if (wave < R) {  // per-head query sum: wave r adds the 128 entries of head r
    const int r = wave;
    float v = 0.f;
    for (int p = lane; p < kD; p += 64)
      v += __half2float(q[((long long)b * L.Hq + hk * R + r) * kD + p]);
    v = wave_sum(v);
    if (lane == 0) {
      sm.qsum[r] = c * v;
      sm.qinit[r] = -1.5f * v * (1.0f / 65536.0f);
    }
  } else if (lane == 0) {
    sm.qinit[wave] = 0.f;
  }
  __syncthreads();

  // A operand of token group g, step st: row i = l%16 belongs to group i/4 and head i%4
  half8_t qop[4][4];
#pragma unroll
  for (int g = 0; g < 4; ++g)
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      half8_t v = *reinterpret_cast<const half8_t *>(sm.qa[lane >> 4][st][lane & 3]);
      if (((lane >> 2) & 3) != g) v = half8_t{0, 0, 0, 0, 0, 0, 0, 0};
      qop[g][st] = v;
    }
  float qsc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) qsc[r] = sm.qsum[r];
  // The score accumulators start at -1.5*sum(q): the products then sum q*(c - 1.5), centred
  // codes, which keeps both halves of  scale*sum q(c-1.5) + (zero+1.5 scale)*sum q  small.
  const float4_t dinit = {sm.qinit[0], sm.qinit[1], sm.qinit[2], sm.qinit[3]};

  // ---- this chunk, this wave's tiles ----
  const long long n_tiles = (nq + 63) >> 6;
  long long tile_begin = (long long)sp * tiles_per_split;
  long long tile_end = tile_begin + tiles_per_split;
  if (tile_end > n_tiles) tile_end = n_tiles;

  const uint8_t *kc = L.k_codes + head * L.Tcap * (kD / 4);
  const float2 *km = reinterpret_cast<const float2 *>(L.k_meta) + head * L.Tcap;
  const float2 *vm = reinterpret_cast<const float2 *>(L.v_meta) + head * L.Tcap;
  const uint8_t *vc = L.v_codes + head * L.n_vblocks * L.v_block_bytes;
  const long long last_blk = (nq - 1) >> 5;
  const int unit_off = TERNARY ? ((13 * lane) & ~3) : 16 * lane;
  const int unit_sh = TERNARY ? ((13 * lane) & 3) : 0;
  // token slot i = lane%8 sits in register m = i/2 at bit {4,6,8,8}[m]: undo 2^(bit-4)
  const float kslot_scale = ((lane >> 1) & 3) == 0 ? 1.f : ((lane >> 1) & 3) == 1 ? 0.25f : 0.0625f;

  float mref[R], lsum[R], zacc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) mref[r] = 0.f, lsum[r] = 0.f, zacc[r] = 0.f;
  float beta = 1.f;
  float4_t acc[8];
#pragma unroll
  for (int n = 0; n < 8; ++n) acc[n] = float4_t{0.f, 0.f, 0.f, 0.f};
  bool first = true;

  for (long long tile = tile_begin + wave; tile < tile_end; tile += 4) {
    const long long t = tile * 64 + lane;
    const bool valid = t < nq;
    const long long tc = valid ? t : nq - 1;
    // ---- loads ----
    uint2_t kq[4];  // lane (j = l%16, kb = l/16): quarter kb of the rows of tokens 16g + j
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      long long tg = tile * 64 + 16 * g + (lane & 15);
      if (tg >= nq) tg = nq - 1;
      kq[g] = *reinterpret_cast<const uint2_t *>(kc + tg * 32 + 8 * (lane >> 4));
    }
    const float2 kmeta = km[tc];
    const float2 vmeta = vm[tc];
    long long blk0 = 2 * tile, blk1 = 2 * tile + 1;
    if (blk1 > last_blk) blk1 = last_blk;
    const Unit16 v0 = *reinterpret_cast<const Unit16 *>(vc + blk0 * L.v_block_bytes + unit_off);
    const Unit16 v1 = *reinterpret_cast<const Unit16 *>(vc + blk1 * L.v_block_bytes + unit_off);

    // ---- scores: 4 token groups x 4 products of 32 channels, one accumulator ----
    float4_t d0 = dinit;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      half8_t bop[4];
      unpack_k(kq[g].x, &bop[0]);
      unpack_k(kq[g].y, &bop[2]);
#pragma unroll
      for (int st = 0; st < 4; ++st)
        d0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(qop[g][st], bop[st], d0, 0, 0, 0);
    }
    // u = log2-domain score minus the running reference
    const float a_t = kmeta.x * (c * 65536.0f);  // codes carry 2^(s-24), the query 2^(8-s)
    const float zc = fmaf(1.5f, kmeta.x, kmeta.y);  // dequantized value of the centre code 1.5
    float u[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float dot = d0[r];
      u[r] = fmaf(dot, a_t, fmaf(zc, qsc[r], -mref[r]));
      if (!valid) u[r] = -INFINITY;
    }
    const float vs = valid ? vmeta.x : 0.f;
    bool trig = vs * beta > kVsLimit;
#pragma unroll
    for (int r = 0; r < R; ++r) trig |= u[r] > kRefSlack;
    if (first || __any(trig)) {
      // move the reference (and the value-scale normalisation) and rescale what is accumulated
      float f[R];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const float umax = wave_max(u[r]);
        const float delta = first ? umax : fmaxf(umax, 0.f);
        f[r] = first ? 0.f : exp2f(-delta);
        mref[r] += delta;
        u[r] -= delta;
        lsum[r] *= f[r];
        zacc[r] *= f[r];
      }
      const float vsmax = wave_max(vs);
      float g = 1.f;
      if (vsmax * beta > kVsTarget || first) {
        float nb = beta;
        if (vsmax > 0.f) {
          int e;
          (void)frexpf(vsmax, &e);            // vsmax = fr * 2^e, fr in [0.5, 1)
          nb = ldexpf(1.f, 8 - e);            // vsmax * nb in [128, 256)
        }
        g = nb / beta;
        beta = nb;
      }
      if (!first) {
        const int col = lane & 15;
        float fc = 0.f;
#pragma unroll
        for (int r = 0; r < R; ++r) fc = (col % R == r) ? f[r] : fc;
        fc *= g;
#pragma unroll
        for (int n = 0; n < 8; ++n) acc[n] *= fc;
      }
      first = false;
    }

    // ---- weights: p = 2^u, P' = p * vscale * beta * 2^(-2m), split into high and low fp16 ----
    const float vsb = vs * beta * kslot_scale;
    _Float16 *pw = &sm.pbuf[wave][lane >> 5][0][lane & 31];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float p = exp2f(u[r]);
      lsum[r] += p;
      zacc[r] = fmaf(p, valid ? vmeta.y : 0.f, zacc[r]);
      const float pp = p * vsb;
      const float hi = __builtin_bit_cast(float, __builtin_bit_cast(unsigned, pp) & 0xffffe000u);
      const float lo = pp - hi;
      pw[r * 32] = (_Float16)hi;
      pw[(R + r) * 32] = (_Float16)lo;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- values: two blocks of 32 tokens, 8 channel tiles each ----
    const int col = lane & 15, kb = lane >> 4;
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      half8_t pop = {0, 0, 0, 0, 0, 0, 0, 0};
      if (col < 2 * R) pop = *reinterpret_cast<const half8_t *>(&sm.pbuf[wave][blk][col][8 * kb]);
      const Unit16 raw = blk ? v1 : v0;
      unsigned fld[8];
      if (TERNARY) {
        const unsigned u0 = __builtin_amdgcn_alignbyte(raw.y, raw.x, unit_sh);
        const unsigned u1 = __builtin_amdgcn_alignbyte(raw.z, raw.y, unit_sh);
        const unsigned u2 = __builtin_amdgcn_alignbyte(raw.w, raw.z, unit_sh);
        const unsigned u3 = raw.w >> (8 * unit_sh);
        unsigned f[8];
        f[0] = u0 & 0x1fffu;
        f[1] = (u0 >> 13) & 0x1fffu;
        f[2] = __builtin_amdgcn_alignbit(u1, u0, 26) & 0x1fffu;
        f[3] = (u1 >> 7) & 0x1fffu;
        f[4] = __builtin_amdgcn_alignbit(u2, u1, 20) & 0x1fffu;
        f[5] = (u2 >> 1) & 0x1fffu;
        f[6] = (u2 >> 14) & 0x1fffu;
        f[7] = __builtin_amdgcn_alignbit(u3, u2, 27) & 0x1fffu;
#pragma unroll
        for (int n = 0; n < 8; ++n) fld[n] = sm.lut[f[n]];
#pragma unroll
        for (int n = 0; n < 8; ++n)
          acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack_v_entry(fld[n]), pop, acc[n], 0, 0, 0);
      } else {
        const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int n = 0; n < 8; ++n) {
          const unsigned f = (n & 1) ? (w[n >> 1] >> 8) : w[n >> 1];
          acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack_v_field(f), pop, acc[n], 0, 0, 0);
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
  }

  // ---- epilogue: fold columns, lanes and the four waves; write this chunk's partial ----
  {
    const int col = lane & 15, kb = lane >> 4;
    const float unscale = 1048576.0f / beta;  // codes carried 2^(4-24)
    if (col < 2 * R) {
#pragma unroll
      for (int n = 0; n < 8; ++n)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) sm.stage[wave][col][16 * n + 4 * kb + rr] = acc[n][rr] * unscale;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float ls = wave_sum(lsum[r]), zs = wave_sum(zacc[r]);
      if (lane == 0) {
        sm.wm[wave][r] = first ? -INFINITY : mref[r];
        sm.wl[wave][r] = ls;
        sm.wz[wave][r] = zs;
      }
    }
  }
  __syncthreads();
  for (int x = tid; x < R * kD; x += 256) {
    const int r = x >> 7, p = x & 127;
    float mstar = fmaxf(fmaxf(sm.wm[0][r], sm.wm[1][r]), fmaxf(sm.wm[2][r], sm.wm[3][r]));
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      if (sm.wl[w][r] > 0.f) {
        const float e = exp2f(sm.wm[w][r] - mstar);
        den += e * sm.wl[w][r];
        num += e * (sm.stage[w][r][p] + sm.stage[w][R + r][p] + sm.wz[w][r]);
      }
    }
    float *part = L.workspace + (((long long)b * L.Hq + hk * R + r) * (SKVQ_MAX_SPLITS + 1) + sp) * kPartialStride;
    part[4 + L.perm_v[hk * kD + p]] = num;
    if (p == 0) {
      part[0] = mstar;
      part[1] = den;
    }
  }
}

}  // namespace

bool decode_mfma_supported(const Layout &L) { return L.G == kD && (L.R == 1 || L.R == 2 || L.R == 4); }

hipError_t launch_decode_mfma(const Layout &L, const __half *q, long long nq, int n_splits,
                              long long tiles_per_split, hipStream_t s) {
  const dim3 grid(n_splits, L.Hk, L.B), block(256);
#define SKVQ_LAUNCH(RR, TT) \
  hipLaunchKernelGGL((decode_mfma_kernel<RR, TT>), grid, block, 0, s, L, q, nq, tiles_per_split)
  const bool ter = L.v_levels == 3;
  switch (L.R) {
    case 1: if (ter) SKVQ_LAUNCH(1, true); else SKVQ_LAUNCH(1, false); break;
    case 2: if (ter) SKVQ_LAUNCH(2, true); else SKVQ_LAUNCH(2, false); break;
    case 4: if (ter) SKVQ_LAUNCH(4, true); else SKVQ_LAUNCH(4, false); break;
    default: return hipErrorInvalidValue;
  }
#undef SKVQ_LAUNCH
  return hipGetLastError();
}

}  // namespace skvq
