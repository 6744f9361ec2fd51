// Matrix-core kernel of skvq_decode_attention for gfx950: packed chunks and the fp16 tokens
// (attention sinks, window) in one launch, one partial per chunk.  Templated on the query
// heads a workgroup serves (1, 2, 4), the K format (2-, 3-, 4-bit), the V format (3-level, 2-, 3-,
// 4-bit), the (scale, zero) format, the groups per head (1, 2, 4) and whether the groups are
// unequal (whole 16-position pieces of the head, mapped to groups by Layout::gmap: then every
// piece has its own score accumulator and weight operand).  This header is compiled
// once per (K format, V format) pair (SKVQ_KL, SKVQ_VL) by skvq_decode_mfma_inst.hip.
// A kv head that is read as one chunk has its output written by that chunk's workgroup; several
// chunks leave partials for merge_kernel.  (Merging them inside this launch was built twice and
// dropped.  With device-scope fences: each fence writes back and invalidates a whole L2, 25 us over
// 256 workgroups.  With all chunks of a kv head on one XCD -- workgroup i of a grid runs on XCD
// i % 8 -- and the hand-off through that XCD's L2 (stores acknowledged, a ticket from an atomic
// counter, the last workgroup reads the partials): correct, and as long as the second launch:
// acknowledgement 0.3 us + ticket 0.8 us + reading and combining 32 partials 1.6 - 2.8 us on the
// slowest workgroup's tail, against 3.0 us for merge_kernel, of which 2.0 us is what any dependent
// launch costs.)
//
// One workgroup of 8 wavefronts per chunk (one per compute unit when the cache is long
// enough).  Per wavefront, per tile of 64 packed tokens:
//   QK   S^T[head][token] by 32 v_mfma_f32_4x4x4_16b_f16 (16 independent 4x4 blocks, lane =
//        token): the B operand is the lane's own 32-byte key row, its 2-bit codes turned into
//        fp16 SUBNORMALS by one AND each (a code c sitting at mantissa bit s is the fp16 value
//        c*2^(s-24)); the A operand is the reordered query, pre-multiplied by the matching
//        power of two, held in registers.  One accumulator per group; afterwards lane l holds
//        the scores of token l for the (up to) four heads.
//   softmax  lazily re-referenced online softmax in the exp2 domain: the running reference m
//        only moves when a score exceeds it by more than 2^6 (wave-uniform branch).
//   PV   O^T[channel][head] by 16 v_mfma_f32_16x16x32_f16: the A operand is the V block unit
//        that the lane loaded (8 tokens x 8 channels, token-minor; a 3-level field is the index
//        of a 16-byte table entry in LDS that IS the operand), the B operand holds p*scale
//        (one per group) split into a high and a low fp16 part (two columns per head) so that
//        the weights keep ~22 bits.
// The zero-points never enter the matrix products: sum_p q_p (s c_p + z) = s sum q c + z sum q
// and sum_t w_t (s_t c + z_t) = sum (w_t s_t) c + sum w_t z_t, per group.
//
// The matrix core accumulates products of subnormal inputs as if their mantissa were full, so
// a code at mantissa bit s costs about (10 - s) bits of the accumulator's precision; every
// 2-bit code is therefore moved to bit 4, 6 or 8 before it is masked out, every 4-bit code to
// bit 4 (its top bit must stay inside the 10 mantissa bits).  A 3-bit code is its two low bits,
// handled like a 2-bit code, with the top bit ORed in two places higher; at mantissa bit 8 that
// top bit is the lowest exponent bit, and the value is still code * 2^(8-24): the fp16 numbers
// 4..7 times 2^-16 are the first normal binade, 2^-14 * (1 + m/4).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <math.h>

#include "skvq_internal.h"
#include "skvq_append_device.h"

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
typedef uint4_t uint4_a4_t __attribute__((aligned(4)));
typedef uint2_t uint2_a4_t __attribute__((aligned(4)));
// Loads of packed cache data.  Every byte is read once per call, so a load may be marked as
// streaming (STREAM): the data then need not displace what the caches hold for longer (the query,
// the permutations, the partials).  That pays where one load instruction takes all that a
// wavefront wants of a cache line soon (32-byte key rows, 13- and 16-byte V units: 4-7 % at long
// contexts); where a row or unit is fetched by several instructions in turn (48- and 64-byte key
// rows, 24- and 32-byte V units) the later ones would miss, and the kernel is 20 % slower: those
// formats load plainly.
template <bool STREAM, class T>
__device__ __forceinline__ T load_as(const T *p) {
  if constexpr (STREAM) return __builtin_nontemporal_load(p); else return *p;
}
template <bool STREAM>
__device__ __forceinline__ uint4_t stream_load(const uint4_t *p) { return load_as<STREAM>(p); }
template <bool STREAM>
__device__ __forceinline__ Unit16 stream_load_unit(const void *p) {
  const uint4_t v = load_as<STREAM>(reinterpret_cast<const uint4_a4_t *>(p));
  return Unit16{v.x, v.y, v.z, v.w};
}
template <bool STREAM>
__device__ __forceinline__ uint2_t stream_load_pair(const void *p) {
  return load_as<STREAM>(reinterpret_cast<const uint2_a4_t *>(p));
}
template <bool STREAM, class T>  // a naturally aligned block of 2, 4, 8, 16 or 32 bytes
__device__ __forceinline__ T stream_load_block(const T *p) {
  if constexpr (sizeof(T) == 2) {
    return __builtin_bit_cast(T, load_as<STREAM>(reinterpret_cast<const unsigned short *>(p)));
  } else if constexpr (sizeof(T) == 4) {
    return __builtin_bit_cast(T, load_as<STREAM>(reinterpret_cast<const unsigned *>(p)));
  } else if constexpr (sizeof(T) == 8) {
    return __builtin_bit_cast(T, load_as<STREAM>(reinterpret_cast<const uint2_t *>(p)));
  } else if constexpr (sizeof(T) == 16) {
    return __builtin_bit_cast(T, load_as<STREAM>(reinterpret_cast<const uint4_t *>(p)));
  } else {
    static_assert(sizeof(T) == 32, "unexpected block size");
    struct Two {
      uint4_t a, b;
    };
    const uint4_t *q = reinterpret_cast<const uint4_t *>(p);
    return __builtin_bit_cast(T, Two{load_as<STREAM>(q), load_as<STREAM>(q + 1)});
  }
}

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kRefSlack = 6.0f;    // scores may exceed the running reference by 2^6
constexpr float kVsTarget = 256.0f;  // max(v scale)*beta is brought below this ...
constexpr float kVsLimit = 512.0f;   // ... and re-normalised when a token exceeds this
constexpr unsigned kM4 = 0x00300030u, kM6 = 0x00c000c0u, kM8 = 0x03000300u;
constexpr unsigned kN4 = 0x00f000f0u;  // a 4-bit code at mantissa bit 4 of each half
constexpr unsigned kB6 = 0x00400040u, kB8 = 0x01000100u, kB10 = 0x04000400u;  // one bit of each half

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Cross-lane moves inside a row of 16 lanes (data-parallel primitives: no LDS round trip).
// A source lane outside the row reads as 0.
template <int CTRL>
__device__ __forceinline__ float row_move(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}
constexpr int kQuadSwap1 = 0xB1;       // quad_perm [1,0,3,2]
constexpr int kQuadSwap2 = 0x4E;       // quad_perm [2,3,0,1]
constexpr int kRowHalfMirror = 0x141;  // lane i reads lane 7 - i of its half row
constexpr int kRowMirror = 0x140;      // lane i reads lane 15 - i of its row
constexpr int kRowShl = 0x100;         // + n: lane i reads lane i + n of its row

// The sum over the 64 lanes, valid in lane 63 only: the row sums as above, then two broadcasts from
// row to row (no lane reads through scalar registers: six dependent moves in all).
__device__ __forceinline__ float wave_sum_in_last_lane(float v) {
  v += row_move<kQuadSwap1>(v);
  v += row_move<kQuadSwap2>(v);
  v += row_move<kRowHalfMirror>(v);
  v += row_move<kRowMirror>(v);  // every lane: the sum of its row
  // lane 15 of rows 0 and 2 to rows 1 and 3; lane 31 to rows 2 and 3 (other rows get 0)
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x142, 0xA, 0xF, false));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x143, 0xC, 0xF, false));
  return v;
}

// The maximum over the 64 lanes as a wave-uniform value: the same moves with maxima (rows that a
// broadcast does not reach keep -inf), then one lane read.  (The median with +inf is the maximum as
// one instruction: fmaxf would first re-canonicalize both operands.)
__device__ __forceinline__ float max_of(float a, float b) { return __builtin_amdgcn_fmed3f(a, b, INFINITY); }
__device__ __forceinline__ float wave_max(float v) {
  v = max_of(v, row_move<kQuadSwap1>(v));
  v = max_of(v, row_move<kQuadSwap2>(v));
  v = max_of(v, row_move<kRowHalfMirror>(v));
  v = max_of(v, row_move<kRowMirror>(v));  // every lane: the maximum of its row
  const int lowest = __builtin_bit_cast(int, -INFINITY);
  v = max_of(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(lowest, __builtin_bit_cast(int, v), 0x142, 0xA, 0xF, false)));
  v = max_of(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(lowest, __builtin_bit_cast(int, v), 0x143, 0xC, 0xF, false)));
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

__device__ __forceinline__ half4_t h4(unsigned a, unsigned b) { return __builtin_bit_cast(half4_t, uint2_t{a, b}); }

// Key dword (16 codes, position e at bit 2e) -> four B operands of the 4x4x4 product.
// Operand x holds positions e = {2x, 2x+8, 2x+1, 2x+9}, at mantissa bits
// {4,4,6,6}, {4,4,6,6}, {8,8,4,4}, {6,6,8,8} for x = 0..3.
__device__ __forceinline__ void unpack_k(unsigned w, half4_t b[4]) {
  const unsigned wl = w << 4, wr = w >> 6;
  b[0] = h4(wl & kM4, wl & kM6);
  b[1] = h4(w & kM4, w & kM6);
  b[2] = h4(w & kM8, wr & kM4);
  b[3] = h4(wr & kM6, wr & kM8);
}

// 3-bit keys: `w` holds the low two bits of 16 codes as a 2-bit dword does, `h` is the plane dword
// with their top bits (DD = 0: w is the even key dword of the pair that shares h, 1: the odd one).
// Same operands as unpack_k; the top bit of a code at mantissa bit s goes to bit s + 2.  The plane's
// bit order makes one shifted copy of h serve three codes.
template <int DD>
__device__ __forceinline__ void unpack_k3(unsigned w, unsigned h, half4_t b[4]) {
  const unsigned wl = w << 4, wr = w >> 6;
  const unsigned ha = DD ? h >> 1 : h << 6;  // positions e = 0, 1, 4 (and e + 8)
  const unsigned hb = DD ? h >> 4 : h << 5;  // e = 2, 3, 7
  const unsigned hc = DD ? h >> 7 : h;       // e = 5, 6
  b[0] = h4((wl & kM4) | (ha & kB6), (wl & kM6) | (ha & kB8));
  b[1] = h4((w & kM4) | (hb & kB6), (w & kM6) | (hb & kB8));
  b[2] = h4((w & kM8) | (ha & kB10), (wr & kM4) | (hc & kB6));
  b[3] = h4((wr & kM6) | (hc & kB8), (wr & kM8) | (hb & kB10));
}

// 4-bit key dword (8 codes, position e at bit 4e) -> two B operands.  Operand y holds positions
// e = {2y, 2y+4, 2y+1, 2y+5}, all at mantissa bit 4.
__device__ __forceinline__ void unpack_k4(unsigned w, half4_t b[2]) {
  b[0] = h4((w << 4) & kN4, w & kN4);
  b[1] = h4((w >> 4) & kN4, (w >> 8) & kN4);
}
// The same bookkeeping as k_slot_of below, for 4-bit rows.
__device__ __forceinline__ void k4_slot_of(int p, int &step, int &kslot, int &shift) {
  const int d = p >> 3, e = p & 7, j = e & 3, hi = e >> 2;  // e = j + 4*hi
  step = 2 * d + (j >> 1);
  kslot = 2 * (j & 1) + hi;
  shift = 4;
}

// For reordered position p: which of the 32 products, which k slot of it, and the mantissa
// bit the key code sits at there.
__device__ __forceinline__ void k_slot_of(int p, int &step, int &kslot, int &shift) {
  const int d = p >> 4, e = p & 15, lo = e & 7, hi = e >> 3;  // e = lo + 8*hi
  step = 4 * d + (lo >> 1);
  kslot = 2 * (lo & 1) + hi;
  const int tab = 0x86486464;  // bit position of code lo (and lo+8), one nibble each
  shift = (tab >> (4 * lo)) & 15;
}

// Eight tokens of one channel -> A operand of the 16x16x32 product: register m holds tokens
// 2m (low half) and 2m+1 (high half); 2-bit units: at mantissa bit {4, 6, 8, 8}[m] (masked out
// of the unit's field), 3-level units: all at bit 8 (read from the table).
// From a 2-bit unit field (pair m at bit 2m of each half; `f` has the field in bits 0..7):
__device__ __forceinline__ half8_t unpack_v_field(unsigned f) {
  const unsigned a = f << 4, b = f << 2;
  return __builtin_bit_cast(half8_t, uint4_t{a & kM4, a & kM6, a & kM8, b & kM8});
}

// From a 3-bit unit: the 2-bit field as above plus the plane dword `h` with the top bits of
// fields 4J .. 4J+3 (NN = the field's index among those four).
template <int NN>
__device__ __forceinline__ half8_t unpack_v3_field(unsigned f, unsigned h) {
  const unsigned a = f << 4, b = f << 2;
  const unsigned ha = NN == 0 ? h << 6 : NN == 1 ? h << 5 : NN == 2 ? h : h >> 1;  // token pairs 0, 1, 2
  const unsigned hb = h >> (2 + NN);                                             // token pair 3
  return __builtin_bit_cast(half8_t, uint4_t{(a & kM4) | (ha & kB6), (a & kM6) | (ha & kB8), (a & kM8) | (ha & kB10),
                                             (b & kM8) | (hb & kB10)});
}

// From a 4-bit unit field (one dword: token pair m at bit 4m of each half), all at bit 4:
__device__ __forceinline__ half8_t unpack_v4_field(unsigned f) {
  return __builtin_bit_cast(half8_t, uint4_t{(f << 4) & kN4, f & kN4, (f >> 4) & kN4, (f >> 8) & kN4});
}

constexpr int kNW = 8;              // wavefronts per workgroup (2 per SIMD: 256 registers each)
constexpr int kThreads = 64 * kNW;
constexpr int kOldShare = 3, kYoungShare = 2;                        // tiles per deal: waves 0..3 / 4..7
constexpr int kDealPeriod = (kNW / 2) * (kOldShare + kYoungShare);  // tiles per deal
constexpr int kAppendLagTiles = 12;  // tiles that the workgroup which also appends the new token is spared
constexpr int kRingWaves = kNW;     // every wavefront of a workgroup may own ring slices
constexpr int kRingSlice = 4;       // ring tokens per slice (the slice code reads four rows of 16 lanes)

constexpr int kCombStride = kD + 16;  // floats; the padding spreads the accumulator columns over the banks

template <int R, bool TERNARY, int NG>
struct Smem {
  // 13-bit field -> the A operand of its eight tokens (104976 bytes, built by the workgroup
  // from the two 81-entry tables: four base-3 digits -> the operand halves of tokens 0..3 / 4..7)
  uint4_t lut[TERNARY ? 6561 : 1];
  uint2_t lut4[TERNARY ? 2 : 1][81];
  // per wave: the weights of the current tile, [block][group][column][token slot]; after the
  // wave's last tile the same bytes stage its O^T, [head][reordered position]
  union WaveBuf {
    _Float16 pbuf[2][NG][2 * R][32];
    float stage[R][kCombStride];
  } wb[kNW];
  float qraw[4][kD];                   // the query heads as loaded (rows >= R are zero)
  _Float16 qa[32][4][4];               // A operands of the score product: [step][head][k slot]
  alignas(16) float qpart[4][8];       // per head: sums of the reordered query over 16 positions each
  alignas(16) float qtotal[4];         // per head: the sum of the whole query (one group per head)
  // epilogue: per-wave running reference, sum of weights, sum of weight*zero, for the packed
  // tiles (w*) and for the ring slices (r*) of the wave
  // ([head][...][wave]: the epilogue reads a head's eight entries as two 16-byte pieces)
  alignas(16) float wm[R][kNW], wl[R][kNW], wz[R][NG][kNW], rm[R][kNW], rl[R][kNW];
  float ring_o[kNW][R][kD];            // per wave: its ring slices' outputs, original channel order
};

// One 4-channel step of the score product.  The A operand of step ST lives in lanes
// 4*(ST%16) .. 4*(ST%16)+3 of register pair ST/16 and is broadcast to all 16 blocks.
template <int ST>
__device__ __forceinline__ float4_t qk_step(half4_t a_lo, half4_t a_hi, half4_t b, float4_t d) {
  if constexpr (ST < 16)
    return __builtin_amdgcn_mfma_f32_4x4x4f16(a_lo, b, d, 4, ST, 0);
  else
    return __builtin_amdgcn_mfma_f32_4x4x4f16(a_hi, b, d, 4, ST - 16, 0);
}
template <int D>
__device__ __forceinline__ float4_t qk_dword(unsigned w, half4_t a_lo, half4_t a_hi, float4_t d) {
  half4_t bop[4];
  unpack_k(w, bop);
  d = qk_step<4 * D + 0>(a_lo, a_hi, bop[0], d);
  d = qk_step<4 * D + 1>(a_lo, a_hi, bop[1], d);
  d = qk_step<4 * D + 2>(a_lo, a_hi, bop[2], d);
  d = qk_step<4 * D + 3>(a_lo, a_hi, bop[3], d);
  return d;
}

template <int D>  // 3-bit keys: dword D of the 2-bit plane and the plane dword of its pair
__device__ __forceinline__ float4_t qk_dword3(unsigned w, unsigned h, half4_t a_lo, half4_t a_hi, float4_t d) {
  half4_t bop[4];
  unpack_k3<D & 1>(w, h, bop);
  d = qk_step<4 * D + 0>(a_lo, a_hi, bop[0], d);
  d = qk_step<4 * D + 1>(a_lo, a_hi, bop[1], d);
  d = qk_step<4 * D + 2>(a_lo, a_hi, bop[2], d);
  d = qk_step<4 * D + 3>(a_lo, a_hi, bop[3], d);
  return d;
}
template <int D>  // D = 0..15: dword of a 4-bit row, positions 8D .. 8D+7
__device__ __forceinline__ float4_t qk_dword4(unsigned w, half4_t a_lo, half4_t a_hi, float4_t d) {
  half4_t bop[2];
  unpack_k4(w, bop);
  d = qk_step<2 * D + 0>(a_lo, a_hi, bop[0], d);
  d = qk_step<2 * D + 1>(a_lo, a_hi, bop[1], d);
  return d;
}

// A stored (scale, zero) pair as one lane loads it, and its value.
template <int META>
struct MetaWord {
  typedef float2 type;
};
template <>
struct MetaWord<SKVQ_META_F16> {
  typedef unsigned type;
};
template <>
struct MetaWord<SKVQ_META_FP8_E4M3> {
  typedef unsigned short type;
};
__device__ __forceinline__ float2 meta_value(float2 w) { return w; }
__device__ __forceinline__ float2 meta_value(unsigned w) {
  const __half2 h = __builtin_bit_cast(__half2, w);
  return make_float2(__low2float(h), __high2float(h));
}
__device__ __forceinline__ float2 meta_value(unsigned short w) {  // FP8 E4M3: conversion is exact
  return make_float2(__builtin_amdgcn_cvt_f32_fp8((int)w, 0), __builtin_amdgcn_cvt_f32_fp8((int)w, 1));
}

// What one wavefront loads for one tile of 64 tokens.
template <int META, int NG>
struct alignas(sizeof(typename MetaWord<META>::type) * NG > 16 ? 16 : sizeof(typename MetaWord<META>::type) * NG)
    MetaBlock {  // the NG pairs of one token
  typename MetaWord<META>::type m[NG];
};
template <int KL, int VL, int META, int NG>
struct TileData {
  // (named members, not arrays: with arrays the compiler keeps copies of the buffers in registers)
  uint4_t k0, k1, k2, k3;            // lane = token: its 32-byte (k0, k1), 48-byte or 64-byte key row
  MetaBlock<META, NG> kmeta, vmeta;  // lane = token: (scale, zero) per group
  Unit16 v00, v01, v10, v11;         // lane = unit of V block 2*tile (v0x) and 2*tile+1 (v1x): 16 or 32 bytes
  uint2_t vt0, vt1;                  // 3-bit units: their 8 bytes of top bits
};

// What one wavefront loads for one slice of 4 fp16 ring tokens.
struct RingData {
  uint4_t k;      // lane (token = l/16, piece = l%16): 8 channels of the token's key row
  unsigned v[4];  // lane = channel pair: the 4 tokens' values of channels 2l, 2l+1
};

// What the host works out once per launch, so that no workgroup spends its first few hundred
// instructions on divisions: the share of the packed tiles per chunk and the ring's first row.
struct ChunkPlan {
  int tiles_q;     // chunk sp holds tiles_q tiles, one more from chunk first_long on: a share of the
  int first_long;  //   tiles plus, when the last chunk's workgroup also appends the new token, the
                   //   kAppendLagTiles it is spared (the last chunk ends at the last tile either way)
  int slot0;       // ring row of the window's oldest token
};

inline ChunkPlan plan_chunks(const Layout &L, long long T, long long nq, int n_sink, int n_splits, bool fused) {
  ChunkPlan p;
  const int n_tiles = (int)((nq + 63) >> 6);
  const int lag = fused && n_tiles >= 4 * kAppendLagTiles * n_splits ? kAppendLagTiles : 0;
  const int nt = n_tiles + lag;
  p.tiles_q = nt / n_splits;
  p.first_long = n_splits - nt % n_splits;
  const long long n_win = (T - nq) - n_sink;
  p.slot0 = (int)((T - n_win) % L.W);
  return p;
}

template <int R, int KL, int VL, int META, int NG, bool UNEQ>
__global__ __launch_bounds__(kThreads, 2) void decode_mfma_kernel(Layout L, const __half *__restrict__ q,
                                                                  long long T, long long nq, int n_sink,
                                                                  int n_splits, int passes, int n_new,
                                                                  const __half *__restrict__ knew,
                                                                  const __half *__restrict__ vnew, long long te,
                                                                  ChunkPlan plan, MergeOut mo) {
  // grid (n_splits, Hk * passes, B): R is the number of query heads one workgroup serves; a kv
  // head with more than four (or with three) query heads is served by `passes` workgroups per
  // chunk, each with R of its L.R query heads (the last one possibly with fewer: the missing
  // heads are computed with a zero query and not stored).
  //   With n_new > 1 query tokens per sequence (the last n_new cached tokens are theirs) the rows
  // of a kv head are its L.R query heads times the n_new tokens, row x = token x / L.R, head
  // x % L.R; query token j does not see the fp16 tokens after its own.
  //   Workgroup sp owns an even share of the packed 64-token tiles of
  // its (sequence, kv head), dealt to its wavefronts round robin, and the ring slices
  // j = sp (mod n_splits), dealt the same way.
  constexpr bool TERNARY = VL == 3, K4 = KL == 16, V4 = VL == 16, K3 = KL == 8, V3 = VL == 8;
  constexpr float kCentre = 0.5f * (KL - 1);  // the key codes enter the products centred
  // score accumulators / weight operands: one per group, or (unequal groups) one per 16 positions
  constexpr int NACC = UNEQ ? 8 : NG;
  __shared__ Smem<R, TERNARY, NG> sm;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int sp = blockIdx.x, by = blockIdx.y;
  const int hk = passes == 1 ? by : by / passes, b = blockIdx.z;
  const unsigned gmap = UNEQ ? L.gmaps[hk] : 0u;
  auto piece_group = [&](int n) { return (int)((gmap >> (4 * n)) & 15u); };  // group of positions 16n..16n+15
  const int head0 = passes == 1 ? 0 : (by % passes) * R;  // first of this workgroup's query heads, within the kv head's
  const long long head = (long long)b * L.Hk + hk;
  const float c = L.sm_scale * kLog2e;

  // ---- the query and the permutations: the first requests of the workgroup, ahead of everything
  //      else (the start-up waits for the query longer than for anything: it queues with the tile
  //      requests of all workgroups) ----
  const int n_rows = n_new * L.R;  // rows of this kv head: (query token, query head)
  // row x of the kv head -> index of its (sequence, query token, query head) in q, the partials and the output
  auto row_index = [&](int x) {
    const int j = n_new == 1 ? 0 : x / L.R;  // (no division on the single-token path)
    return ((long long)b * n_new + j) * L.Hq + hk * L.R + (x - j * L.R);
  };
  __half2 q2 = __floats2half2_rn(0.f, 0.f);
  if (tid < 64 * R && head0 + (tid >> 6) < n_rows)
    q2 = reinterpret_cast<const __half2 *>(q + row_index(head0 + (tid >> 6)) * kD)[lane];
  // (staging: wavefront w < 4 places head w's query at the positions lane and 64 + lane)
  const int pk0 = L.perm_k[hk * kD + lane], pk1 = L.perm_k[hk * kD + 64 + lane];
  const int pv_ch = L.perm_v[hk * kD + (tid & 127)];  // for the epilogue: channel of position tid%128

  // ---- the new token taken along (knew != null; one query token, passes == 1, and the token
  //      that leaves the window, if any, is packed: the host sees to that).  T counts the new
  //      token.  The workgroup of the last chunk does what the append kernel does (its tiles are
  //      the only ones that read the packed row, the V block and the metadata that this writes;
  //      nobody reads the ring slot: the new token's row is taken from knew / vnew below).  Its
  //      stores have completed, in this compute unit's own cache order, before its first tile
  //      load is issued, and no load of the branch is pending where the paths join. ----
  const bool fused = knew != nullptr;
  if (fused && sp == n_splits - 1) {
    append_token(L, knew, vnew, T - 1, -1, te, hk, b, wave, lane, reinterpret_cast<__half(*)[kD]>(&sm.ring_o[0][0][0]),
                 reinterpret_cast<uint8_t *>(&sm.ring_o[0][0][0]) + 2 * kD * sizeof(__half));
    __threadfence_block();
    // (the fence alone need not wait for the stores.  The builtin, not inline assembly: the
    // compiler then knows that no load of this branch is pending, and adds no wait for one to
    // the common path below.)  vmcnt(0), the other counters left alone
    __builtin_amdgcn_s_waitcnt(0x0F70);
    asm volatile("" ::: "memory");
    __syncthreads();
  }

  // ---- this chunk, this wave's tiles ----
  // (with the new token taken along the last chunk is shorter by about the time its workgroup
  // spends on the append)
  const int n_tiles = (int)((nq + 63) >> 6);
  // (the later chunks hold the odd tiles: the last chunk is never empty while there is a tile,
  // and the tile of the token that leaves the window is always its own)
  const int n_long = sp > plan.first_long ? sp - plan.first_long : 0;  // longer chunks before this one
  const int tile_begin = sp * plan.tiles_q + n_long;
  const int tile_end = sp == n_splits - 1 ? n_tiles : tile_begin + plan.tiles_q + (sp >= plan.first_long ? 1 : 0);

  constexpr int kRowBytes = K4 ? 64 : K3 ? 48 : 32;
  const uint8_t *kc = L.k_codes + head * L.Tcap * kRowBytes;
  typedef TileData<KL, VL, META, NG> Tile;
  typedef MetaBlock<META, NG> meta_block;
  const meta_block *km = reinterpret_cast<const meta_block *>(L.k_meta) + head * L.Tcap;
  const meta_block *vm = reinterpret_cast<const meta_block *>(L.v_meta) + head * L.Tcap;
  const uint8_t *vc = L.v_codes + head * L.n_vblocks * L.v_block_bytes;
  const int last_token = (int)(nq - 1);  // -1 when nothing is packed (then there are no tiles)
  const int last_blk = last_token >> 5;
  const int vbb = TERNARY ? kTernaryBlockBytes : V4 ? kFourBitBlockBytes : V3 ? kThreeBitBlockBytes : kTwoBitBlockBytes;
  const unsigned unit_off = TERNARY ? ((13 * lane) & ~3) : V4 ? 32 * lane : V3 ? 24 * lane : 16 * lane;
  const int unit_sh = TERNARY ? ((13 * lane) & 3) : 0;
  // 2-bit units: token slot i = lane%8 sits in register m = i/2 at bit {4,6,8,8}[m]: undo
  // 2^(bit-4).  3-level units: every slot at bit 8.  4-bit units: every slot at bit 4.
  const float kslot_scale =
      (TERNARY || V4) ? 1.f : ((lane >> 1) & 3) == 0 ? 1.f : ((lane >> 1) & 3) == 1 ? 0.25f : 0.0625f;

  // Loads are issued unconditionally (a tile index past the end is redirected to the last
  // tile, whose lines are in cache by then, and the data is ignored): the compiler can then
  // count the loads in flight and wait for exactly the ones a tile needs.
  const int safe_last_tile = n_tiles > 0 ? n_tiles - 1 : 0;
  const int safe_last_token = last_token > 0 ? last_token : 0;
  const int safe_last_blk = last_blk > 0 ? last_blk : 0;
  // which of the streams are marked as streaming loads (see load_as)
  constexpr bool kStreamK = KL == 4, kStreamV = VL == 3 || VL == 4;
  // (a tile index past the workgroup's share is redirected to tile_cap, the share's last tile, or tile
  // 0 of an empty cache, by the callers: one scalar minimum per load)
  const int tile_cap = max(min(tile_end - 1, safe_last_tile), 0);
  auto load_tile = [&](const int tile) {
    Tile d;
    // every address is a wave-uniform base (the tile's first row, its two V blocks) plus a 32-bit lane
    // offset: the bases are scalar arithmetic, the offsets cost one vector instruction per stream
    // (lanes past the last token -- only in the last tile, masked below -- repeat its row)
    const int rows_here = safe_last_token - tile * 64;  // >= 0
    const unsigned row = min((unsigned)lane, (unsigned)rows_here);
    const uint8_t *kt = kc + (size_t)tile * (64 * kRowBytes);
    const uint8_t *krow = kt + row * (unsigned)kRowBytes;
    d.k0 = stream_load<kStreamK>(reinterpret_cast<const uint4_t *>(krow));
    d.k1 = stream_load<kStreamK>(reinterpret_cast<const uint4_t *>(krow + 16));
    if constexpr (K4) {
      d.k2 = stream_load<kStreamK>(reinterpret_cast<const uint4_t *>(krow + 32));
      d.k3 = stream_load<kStreamK>(reinterpret_cast<const uint4_t *>(krow + 48));
    }
    if constexpr (K3) d.k2 = stream_load<kStreamK>(reinterpret_cast<const uint4_t *>(krow + 32));
    const unsigned moff = row * (unsigned)sizeof(meta_block);
    d.kmeta = stream_load_block<kStreamK>(reinterpret_cast<const meta_block *>(
        reinterpret_cast<const uint8_t *>(km + (size_t)tile * 64) + moff));
    d.vmeta = stream_load_block<kStreamK>(reinterpret_cast<const meta_block *>(
        reinterpret_cast<const uint8_t *>(vm + (size_t)tile * 64) + moff));
    const int blk0 = 2 * tile > safe_last_blk ? safe_last_blk : 2 * tile;
    const int blk1 = blk0 + 1 > safe_last_blk ? safe_last_blk : blk0 + 1;
    const uint8_t *vb0 = vc + (size_t)blk0 * vbb, *vb1 = vc + (size_t)blk1 * vbb;
    // (the lane's offset is hidden from the compiler here: seen as loop-invariant it is folded into a
    // 64-bit vector base once, and every tile then pays vector multiply-adds for the block's address)
    unsigned uoff = unit_off;
    asm("" : "+v"(uoff));
    d.v00 = stream_load_unit<kStreamV>(vb0 + uoff);
    d.v10 = stream_load_unit<kStreamV>(vb1 + uoff);
    if constexpr (V3) {
      d.vt0 = stream_load_pair<kStreamV>(vb0 + uoff + 16);
      d.vt1 = stream_load_pair<kStreamV>(vb1 + uoff + 16);
    }
    if constexpr (V4) {
      d.v01 = stream_load_unit<kStreamV>(vb0 + uoff + 16);
      d.v11 = stream_load_unit<kStreamV>(vb1 + uoff + 16);
    }
    return d;
  };

  // ---- the fp16 ring: slices of 4 tokens, slice j belongs to workgroup j % n_splits and to
  //      the wave whose rank is (j / n_splits) % kRingWaves ----
  // The fp16 tokens in token order: the n_sink sink rows (rows W.. of the ring buffers), then
  // the window's tokens.
  const int n_win = (int)(T - nq) - n_sink, W = L.W;
  const int n_fp = n_sink + n_win;
  const int n_slices = (n_fp + kRingSlice - 1) / kRingSlice;
  const int ring_stride = n_splits * kRingWaves;
  // the younger waves (which get fewer tiles) are first in line for ring slices
  const int ring_rank = (wave + kNW / 2) % kNW;
  const int ring_first = sp + n_splits * ring_rank;
  const bool ring_owner = ring_first < n_slices;
  const int slot0 = plan.slot0;  // ring row of the window's oldest token
  const __half *kwin = L.k_win + head * (W + L.S) * kD;
  const __half *vwin = L.v_win + head * (W + L.S) * kD;
  // (ring token t, clamped to the last one, sits in sink row W + t if it is a sink, else in ring
  // slot slot0 + t - n_sink modulo W; the newest token's row is the caller's when it is taken along)
  auto load_ring = [&](int slice) {
    RingData d;
    // Lane (token l/16 of the slice, piece l%16) works out the row of its own token with vector
    // arithmetic (the same for every slice: no scalar branches per row); the four value rows take
    // theirs from lanes 0, 16, 32 and 48.
    const int t = min(slice * kRingSlice + (lane >> 4), n_fp - 1);
    const int s = slot0 + t - n_sink;
    const int slot = t < n_sink ? W + t : (s >= W ? s - W : s);
    const int fresh = fused && t >= n_fp - 1 ? 1 : 0;  // the caller's row of the new token
    const unsigned row_bytes = (unsigned)slot * (unsigned)(kD * sizeof(__half));
    const char *krow = fresh ? reinterpret_cast<const char *>(knew + head * kD)
                             : reinterpret_cast<const char *>(kwin) + row_bytes;
    d.k = reinterpret_cast<const uint4_t *>(krow)[lane & 15];
#pragma unroll
    for (int k = 0; k < kRingSlice; ++k) {
      const unsigned vb = (unsigned)__builtin_amdgcn_readlane((int)row_bytes, 16 * k);
      const char *vrow = __builtin_amdgcn_readlane(fresh, 16 * k) ? reinterpret_cast<const char *>(vnew + head * kD)
                                                                   : reinterpret_cast<const char *>(vwin) + vb;
      d.v[k] = reinterpret_cast<const unsigned *>(vrow)[lane];
    }
    return d;
  };

  // ---- prologue: one memory round trip.  The small loads (query and permutations above, ring
  //      slice here) are issued BEFORE the tile loads: loads return in order, so the staging below
  //      only has to wait for them and not for the two tiles of packed data behind them. ----
  RingData ring = {};
  if (ring_owner) ring = load_ring(ring_first);  // landed before the tile loop either way (see below)
  asm volatile("" ::: "memory");
  // three tile buffers used in turn (no register copies): while one tile is computed the
  // next two are in flight
  // The two wavefronts of a SIMD do not share it evenly: the older one (waves 0..3) is served
  // first and gets through about three tiles while the younger one gets through two.  The
  // tiles are dealt in that ratio (per 20 tiles: three to each older, two to each younger
  // wave) so that both finish together.
  const int share = wave < kNW / 2 ? kOldShare : kYoungShare;
  const int deal_base = wave < kNW / 2 ? wave : kOldShare * (kNW / 2) + (wave - kNW / 2);
  auto tile_of = [&](int n) {  // n-th tile of this wave
    const int r = n / share;
    return tile_begin + kDealPeriod * r + deal_base + (kNW / 2) * (n - share * r);
  };
  int n_a = 0, n_b = 1, n_c = 2;
  int tile_a = tile_of(n_a), tile_b = tile_of(n_b), tile_c = tile_of(n_c);
  Tile buf_a, buf_b, buf_c;
  buf_a = load_tile(min(tile_a, tile_cap));
  if (TERNARY) {
    // While the loads are in flight the workgroup builds the table: entry f (a base-3 number of
    // eight digits, digit i = code of token i) is the operand itself, register m = codes of
    // tokens 2m (low half) and 2m+1 (high half) as fp16 subnormals c * 2^(8-24).
    if (tid < 162) {
      const int half = tid >= 81, x = half ? tid - 81 : tid;
      const unsigned d0 = x % 3, d1 = (x / 3) % 3, d2 = (x / 9) % 3, d3 = x / 27;
      sm.lut4[half][x] = uint2_t{(d0 << 8) | (d1 << 24), (d2 << 8) | (d3 << 24)};
    }
    __syncthreads();
    // Thread t < 486 keeps the low half of its entries (digits t % 81) and walks through every
    // sixth high half from t / 81 on: one read per entry instead of two, all reads first, then
    // all writes (one LDS latency, not one per entry).
    constexpr int kWalk = 6, kSteps = (81 + kWalk - 1) / kWalk;
    const unsigned first_hi = tid / 81u, lo = tid - 81u * first_hi;
    if (first_hi < kWalk) {
      const uint2_t lo4 = sm.lut4[0][lo];
      uint2_t hi4[kSteps];
#pragma unroll
      for (int i = 0; i < kSteps; ++i) hi4[i] = sm.lut4[1][min(first_hi + kWalk * i, 80u)];
#pragma unroll
      for (int i = 0; i < kSteps; ++i) {
        const unsigned hi = first_hi + kWalk * i;
        if (hi < 81u) sm.lut[81u * hi + lo] = uint4_t{lo4.x, lo4.y, hi4[i].x, hi4[i].y};
      }
    }
  }
  {
    asm volatile("" ::: "memory");
    buf_b = load_tile(min(tile_b, tile_cap));
    // Wavefront w < 4 stages head w by itself: it parks the head's query in LDS as loaded (for the
    // fp16 slices later), reads it back through the permutation (its own writes: no barrier, the
    // LDS serves a wavefront's operations in order) and writes the head's matrix operands and piece
    // sums.  One barrier then covers the operands, the sums and the table.
    if (tid < 256) {
      sm.qraw[wave][2 * lane] = __low2float(q2);
      sm.qraw[wave][2 * lane + 1] = __high2float(q2);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      float both = 0.f;  // the lane's two positions
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int row = wave, p = lane + 64 * j;
        int step, kslot, shift;
        if (K4)
          k4_slot_of(p, step, kslot, shift);
        else
          k_slot_of(p, step, kslot, shift);
        const float x = sm.qraw[row][j ? pk1 : pk0];
        sm.qa[step][row][kslot] = (_Float16)ldexpf(x, 8 - shift);  // exact: a power of two
        both += x;
        if constexpr (UNEQ || NG > 1) {
          // sum of the reordered query over the 16 positions of this row of lanes
          float s16 = x;
          s16 += row_move<kQuadSwap1>(s16);
          s16 += row_move<kQuadSwap2>(s16);
          s16 += row_move<kRowHalfMirror>(s16);
          s16 += row_move<kRowMirror>(s16);
          if ((lane & 15) == 0) sm.qpart[row][p >> 4] = s16;
        }
      }
      if constexpr (!UNEQ && NG == 1) {
        // one group per head: the head's whole sum, formed here once instead of by every wavefront
        both = wave_sum_in_last_lane(both);
        if (lane == 63) sm.qtotal[wave] = both;
      }
    }
    __syncthreads();
  }
  // lane l supplies row l%4 (= head) of step l/4 (first register pair) and 16 + l/4 (second)
  const half4_t qop_lo = *reinterpret_cast<const half4_t *>(sm.qa[lane >> 2][lane & 3]);
  const half4_t qop_hi = *reinterpret_cast<const half4_t *>(sm.qa[16 + (lane >> 2)][lane & 3]);
  // Per group: sm_scale*log2(e) * sum of the reordered query (qsc), and the start value of the
  // score accumulators, -centre*sum(q) in the product's units (2^-16), centre = 1.5 (2-bit) or 7.5
  // (4-bit): the products then sum q*(c - centre), centred codes, which keeps both halves of
  // scale*sum q(c-centre) + (zero+centre*scale)*sum q  small.
  float qsc[R][NG];
  float4_t dinit[UNEQ ? 1 : NG];
  float qp[4][8];  // the piece sums of the four heads (two 16-byte reads per head)
  if constexpr (UNEQ || NG > 1) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float4_t lo4 = *reinterpret_cast<const float4_t *>(&sm.qpart[r][0]);
      const float4_t hi4 = *reinterpret_cast<const float4_t *>(&sm.qpart[r][4]);
#pragma unroll
      for (int x = 0; x < 4; ++x) qp[r][x] = lo4[x], qp[r][4 + x] = hi4[x];
    }
  }
  if constexpr (!UNEQ && NG == 1) {
    const float4_t tot = *reinterpret_cast<const float4_t *>(&sm.qtotal[0]);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (r < R) qsc[r][0] = c * tot[r];
      dinit[0][r] = -kCentre * tot[r] * (1.0f / 65536.0f);
    }
  } else if constexpr (UNEQ) {
    // (a piece's accumulator sums only 16 products: it starts from zero, uncentred)
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
      for (int r = 0; r < R; ++r) {
        float sum = 0.f;
#pragma unroll
        for (int x = 0; x < 8; ++x) sum += piece_group(x) == g ? qp[r][x] : 0.f;
        qsc[r][g] = c * sum;
      }
    dinit[0] = float4_t{0.f, 0.f, 0.f, 0.f};
  } else {
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float sum = 0.f;
#pragma unroll
        for (int x = 0; x < 8 / NG; ++x) sum += qp[r][g * (8 / NG) + x];
        if (r < R) qsc[r][g] = c * sum;
        dinit[g][r] = -kCentre * sum * (1.0f / 65536.0f);
      }
  }

  // ---- ring slices of this wave (plain vector arithmetic, wave-local) ----
  if (ring_owner) {
    float rm[R], rl[R], ro[R][2];  // reference, sum of weights, outputs
#pragma unroll
    for (int r = 0; r < R; ++r) rm[r] = -INFINITY, rl[r] = 0.f, ro[r][0] = ro[r][1] = 0.f;
    // query token j sees the fp16 tokens up to its own, index n_fp - n_new + j (all of them if n_new = 1)
    int ring_last[R];
#pragma unroll
    for (int r = 0; r < R; ++r) ring_last[r] = n_new == 1 ? n_fp - 1 : n_fp - n_new + (head0 + r) / L.R;
    auto ring_slice = [&](const RingData &rd, const int slice) {
      const int tk = lane >> 4, pc = lane & 15;  // token of the slice, 8-channel piece of its row
      const int tok = slice * kRingSlice + tk;  // index among the fp16 tokens
      const bool valid = tok < n_fp;
      const half8_t x = __builtin_bit_cast(half8_t, rd.k);
      float p[R][kRingSlice];  // the four tokens' weights, wave-uniform
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const float4_t qa = *reinterpret_cast<const float4_t *>(&sm.qraw[r][8 * pc]);
        const float4_t qb = *reinterpret_cast<const float4_t *>(&sm.qraw[r][8 * pc + 4]);
        float s = qa[0] * (float)x[0];
        s = fmaf(qa[1], (float)x[1], s);
        s = fmaf(qa[2], (float)x[2], s);
        s = fmaf(qa[3], (float)x[3], s);
        s = fmaf(qb[0], (float)x[4], s);
        s = fmaf(qb[1], (float)x[5], s);
        s = fmaf(qb[2], (float)x[6], s);
        s = fmaf(qb[3], (float)x[7], s);
        s += row_move<kQuadSwap1>(s);
        s += row_move<kQuadSwap2>(s);
        s += row_move<kRowHalfMirror>(s);
        s += row_move<kRowMirror>(s);  // all sixteen lanes of a token now hold its score
        s = valid && tok <= ring_last[r] ? c * s : -INFINITY;
        float sk[kRingSlice];  // the four tokens' scores, read from one lane of each row
#pragma unroll
        for (int k = 0; k < kRingSlice; ++k)
          sk[k] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, s), 16 * k));
        const float mnew = fmaxf(rm[r], fmaxf(fmaxf(sk[0], sk[1]), fmaxf(sk[2], sk[3])));
        // (a query token of a multi-token call may see none of a slice's tokens, nor of the earlier
        // ones: then everything stays zero; -inf minus -inf must not be formed)
        const float mref = mnew == -INFINITY ? 0.f : mnew;
        const float f = fast_exp2(rm[r] - mref);  // 0 for the first slice
#pragma unroll
        for (int k = 0; k < kRingSlice; ++k) p[r][k] = fast_exp2(sk[k] - mref);  // 0 for tokens past the end
        rl[r] = rl[r] * f + (p[r][0] + p[r][1]) + (p[r][2] + p[r][3]);
        ro[r][0] *= f;
        ro[r][1] *= f;
        rm[r] = mnew;
      }
#pragma unroll
      for (int k = 0; k < kRingSlice; ++k) {
        const __half2 v2 = __builtin_bit_cast(__half2, rd.v[k]);
        const float vx = __low2float(v2), vy = __high2float(v2);
#pragma unroll
        for (int r = 0; r < R; ++r) {
          ro[r][0] = fmaf(p[r][k], vx, ro[r][0]);
          ro[r][1] = fmaf(p[r][k], vy, ro[r][1]);
        }
      }
    };
    if (ring_first + ring_stride >= n_slices) {
      // one slice (the usual case): its data was requested before the tile loads
      ring_slice(ring, ring_first);
    } else {
      // several slices: each next one is requested while the current one is computed; those
      // requests queue behind the tile loads, and all of them have landed when this ends
      for (int slice = ring_first; slice < n_slices; slice += ring_stride) {
        RingData ring_next = ring;
        if (slice + ring_stride < n_slices) ring_next = load_ring(slice + ring_stride);
        ring_slice(ring, slice);
        ring = ring_next;
      }
      asm volatile("" ::"v"(ring.k.x), "v"(ring.k.y), "v"(ring.k.z), "v"(ring.k.w), "v"(ring.v[0]),
                   "v"(ring.v[1]), "v"(ring.v[2]), "v"(ring.v[3]));
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      sm.ring_o[wave][r][2 * lane] = ro[r][0];
      sm.ring_o[wave][r][2 * lane + 1] = ro[r][1];
      if (lane == 0) sm.rm[r][wave] = rm[r], sm.rl[r][wave] = rl[r];
    }
  } else if (lane < R) {
    sm.rm[lane][wave] = -INFINITY;
    sm.rl[lane][wave] = 0.f;
  }
  // (No ring load younger than the tile loads may be pending here: it would turn every wait
  // inside the tile loop into a wait for all loads.)

  float mref[R], lsum[R], zacc[R][NG];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    mref[r] = 0.f, lsum[r] = 0.f;
#pragma unroll
    for (int g = 0; g < NG; ++g) zacc[r][g] = 0.f;
  }
  float beta = 1.f, vs_limit = kVsLimit;
  float minus_one = -1.0f;
  asm("" : "+v"(minus_one));
  float4_t acc[8];
#pragma unroll
  for (int n = 0; n < 8; ++n) acc[n] = float4_t{0.f, 0.f, 0.f, 0.f};
  bool first = true;

  auto compute_tile = [&](const Tile &cur, const int tile) {
    const bool valid = tile * 64 + lane <= last_token;

    // ---- scores: 32 products of 4 channels each, one accumulator per group ----
    float4_t dg[NACC];
#pragma unroll
    for (int g = 0; g < NACC; ++g) dg[g] = UNEQ ? float4_t{0.f, 0.f, 0.f, 0.f} : dinit[g];
    if constexpr (K4) {
#define SKVQ_QK4(Q, C, DW) dg[(DW) * NACC / 16] = qk_dword4<DW>(cur.k##Q.C, qop_lo, qop_hi, dg[(DW) * NACC / 16])
      SKVQ_QK4(0, x, 0);  SKVQ_QK4(0, y, 1);  SKVQ_QK4(0, z, 2);  SKVQ_QK4(0, w, 3);
      SKVQ_QK4(1, x, 4);  SKVQ_QK4(1, y, 5);  SKVQ_QK4(1, z, 6);  SKVQ_QK4(1, w, 7);
      SKVQ_QK4(2, x, 8);  SKVQ_QK4(2, y, 9);  SKVQ_QK4(2, z, 10); SKVQ_QK4(2, w, 11);
      SKVQ_QK4(3, x, 12); SKVQ_QK4(3, y, 13); SKVQ_QK4(3, z, 14); SKVQ_QK4(3, w, 15);
#undef SKVQ_QK4
    } else if constexpr (K3) {
      dg[0 * NACC / 8] = qk_dword3<0>(cur.k0.x, cur.k2.x, qop_lo, qop_hi, dg[0 * NACC / 8]);
      dg[1 * NACC / 8] = qk_dword3<1>(cur.k0.y, cur.k2.x, qop_lo, qop_hi, dg[1 * NACC / 8]);
      dg[2 * NACC / 8] = qk_dword3<2>(cur.k0.z, cur.k2.y, qop_lo, qop_hi, dg[2 * NACC / 8]);
      dg[3 * NACC / 8] = qk_dword3<3>(cur.k0.w, cur.k2.y, qop_lo, qop_hi, dg[3 * NACC / 8]);
      dg[4 * NACC / 8] = qk_dword3<4>(cur.k1.x, cur.k2.z, qop_lo, qop_hi, dg[4 * NACC / 8]);
      dg[5 * NACC / 8] = qk_dword3<5>(cur.k1.y, cur.k2.z, qop_lo, qop_hi, dg[5 * NACC / 8]);
      dg[6 * NACC / 8] = qk_dword3<6>(cur.k1.z, cur.k2.w, qop_lo, qop_hi, dg[6 * NACC / 8]);
      dg[7 * NACC / 8] = qk_dword3<7>(cur.k1.w, cur.k2.w, qop_lo, qop_hi, dg[7 * NACC / 8]);
    } else {
      dg[0 * NACC / 8] = qk_dword<0>(cur.k0.x, qop_lo, qop_hi, dg[0 * NACC / 8]);
      dg[1 * NACC / 8] = qk_dword<1>(cur.k0.y, qop_lo, qop_hi, dg[1 * NACC / 8]);
      dg[2 * NACC / 8] = qk_dword<2>(cur.k0.z, qop_lo, qop_hi, dg[2 * NACC / 8]);
      dg[3 * NACC / 8] = qk_dword<3>(cur.k0.w, qop_lo, qop_hi, dg[3 * NACC / 8]);
      dg[4 * NACC / 8] = qk_dword<4>(cur.k1.x, qop_lo, qop_hi, dg[4 * NACC / 8]);
      dg[5 * NACC / 8] = qk_dword<5>(cur.k1.y, qop_lo, qop_hi, dg[5 * NACC / 8]);
      dg[6 * NACC / 8] = qk_dword<6>(cur.k1.z, qop_lo, qop_hi, dg[6 * NACC / 8]);
      dg[7 * NACC / 8] = qk_dword<7>(cur.k1.w, qop_lo, qop_hi, dg[7 * NACC / 8]);
    }
    // u = log2-domain score minus the running reference
    float u[R];
#pragma unroll
    for (int r = 0; r < R; ++r) u[r] = -mref[r];
    if constexpr (UNEQ) {
      float a_t[NG];
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        const float2 kmeta = meta_value(cur.kmeta.m[g]);
        a_t[g] = kmeta.x * (c * 65536.0f);
#pragma unroll
        for (int r = 0; r < R; ++r) u[r] = fmaf(kmeta.y, qsc[r][g], u[r]);  // zero-point * sum of the query
      }
#pragma unroll
      for (int x = 0; x < 8; ++x) {  // each 16-position piece times the scale of its group
        const int g = piece_group(x);
        float a = a_t[0];
#pragma unroll
        for (int y = 1; y < NG; ++y) a = g == y ? a_t[y] : a;
#pragma unroll
        for (int r = 0; r < R; ++r) u[r] = fmaf(dg[x][r], a, u[r]);
      }
    } else {
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        const float2 kmeta = meta_value(cur.kmeta.m[g]);
        const float a_t = kmeta.x * (c * 65536.0f);       // codes carry 2^(s-24), the query 2^(8-s)
        const float zc = fmaf(kCentre, kmeta.x, kmeta.y);  // dequantized value of the centre code
#pragma unroll
        for (int r = 0; r < R; ++r) u[r] = fmaf(dg[g][r], a_t, fmaf(zc, qsc[r][g], u[r]));
      }
    }
    float vs[NG], vz[NG], vs_top = 0.f;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const float2 vmeta = meta_value(cur.vmeta.m[g]);
      vs[g] = vmeta.x, vz[g] = vmeta.y;
    }
    if (tile * 64 + 63 > last_token) {  // (a scalar condition) only the cache's last tile has tokens to drop
#pragma unroll
      for (int g = 0; g < NG; ++g) vs[g] = valid ? vs[g] : 0.f, vz[g] = valid ? vz[g] : 0.f;
#pragma unroll
      for (int r = 0; r < R; ++r)
        if (!valid) u[r] = -INFINITY;
    }
    // (scales are not negative: one group's scale is the largest as it is)
    vs_top = vs[0];
#pragma unroll
    for (int g = 1; g < NG; ++g) vs_top = fmaxf(vs_top, vs[g]);
    // one comparison for the heads' scores (their maximum) and one for the value scale, against
    // the limit divided by beta (a power of two: the same decision as the product against the limit)
    float u_top = u[0];
#pragma unroll
    for (int r = 1; r < R; ++r) u_top = fmaxf(u_top, u[r]);
    const bool trig = (vs_top > vs_limit) | (u_top > kRefSlack);
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
#pragma unroll
        for (int g = 0; g < NG; ++g) zacc[r][g] *= f[r];
      }
      const float vsmax = wave_max(vs_top);
      float g = 1.f;
      if (vsmax * beta > kVsTarget || first) {
        float nb = beta;
        if (vsmax > 0.f) {
          int e;
          (void)frexpf(vsmax, &e);  // vsmax = fr * 2^e, fr in [0.5, 1)
          nb = ldexpf(1.f, 8 - e);  // vsmax * nb in [128, 256)
        }
        g = nb / beta;
        beta = nb;
        vs_limit = kVsLimit / nb;
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

    // ---- weights: p = 2^u, P' = p * vscale * beta * 2^-(bit-4), split into high and low fp16 ----
    const float bk = beta * kslot_scale;
    _Float16 *pw = &sm.wb[wave].pbuf[lane >> 5][0][0][lane & 31];
    // (the high part is the weight converted to fp16 toward zero, two heads per instruction; the
    // low part the fp32 weight minus that fp16 number -- exact -- rounded to fp16 once, as one
    // mixed-precision multiply-add: minus_one is -1 in a form the compiler does not see through)
    float pr[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      pr[r] = fast_exp2(u[r]);
      lsum[r] += pr[r];
    }
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const float vsb = vs[g] * bk;
#pragma unroll
      for (int r = 0; r < R; r += 2) {
        const float pa = pr[r] * vsb, pb = r + 1 < R ? pr[r + 1] * vsb : 0.f;
        const auto hi = __builtin_amdgcn_cvt_pkrtz(pa, pb);
        zacc[r][g] = fmaf(pr[r], vz[g], zacc[r][g]);
        pw[(g * 2 * R + r) * 32] = hi[0];
        pw[(g * 2 * R + R + r) * 32] = (_Float16)__builtin_fmaf((float)hi[0], minus_one, pa);
        if (r + 1 < R) {
          zacc[r + 1][g] = fmaf(pr[r + 1], vz[g], zacc[r + 1][g]);
          pw[(g * 2 * R + r + 1) * 32] = hi[1];
          pw[(g * 2 * R + R + r + 1) * 32] = (_Float16)__builtin_fmaf((float)hi[1], minus_one, pb);
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- values: two blocks of 32 tokens, 8 channel tiles each ----
    const int col = lane & 15, kb = lane >> 4;
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      half8_t pop[NACC];  // the weights (B operand) of each group (or piece) of channel tiles
#pragma unroll
      for (int x = 0; x < NACC; ++x) {
        const int g = UNEQ ? piece_group(x) : x;
        // (columns from 2R on re-read the first ones: nobody reads their results, and an
        // unconditional read needs neither a zeroed operand nor a change of the execution mask)
        pop[x] = *reinterpret_cast<const half8_t *>(&sm.wb[wave].pbuf[blk][g][col % (2 * R)][8 * kb]);
      }
      const Unit16 raw = blk ? cur.v10 : cur.v00;
      if constexpr (V4) {
        const Unit16 raw2 = blk ? cur.v11 : cur.v01;
        const unsigned w[8] = {raw.x, raw.y, raw.z, raw.w, raw2.x, raw2.y, raw2.z, raw2.w};
#pragma unroll
        for (int n = 0; n < 8; ++n)
          acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack_v4_field(w[n]), pop[n * NACC / 8], acc[n], 0, 0, 0);
      } else if (TERNARY) {
        const unsigned u0 = __builtin_amdgcn_alignbyte(raw.y, raw.x, unit_sh);
        const unsigned u1 = __builtin_amdgcn_alignbyte(raw.z, raw.y, unit_sh);
        const unsigned u2 = __builtin_amdgcn_alignbyte(raw.w, raw.z, unit_sh);
        const unsigned u3 = raw.w >> (8 * unit_sh);
        // byte offsets into the table (field * 16), two operations per field
        unsigned f[8];
        f[0] = (u0 << 4) & 0x1fff0u;
        f[1] = (u0 >> 9) & 0x1fff0u;
        f[2] = __builtin_amdgcn_alignbit(u1, u0, 22) & 0x1fff0u;
        f[3] = (u1 >> 3) & 0x1fff0u;
        f[4] = __builtin_amdgcn_alignbit(u2, u1, 16) & 0x1fff0u;
        f[5] = (u2 << 3) & 0x1fff0u;
        f[6] = (u2 >> 10) & 0x1fff0u;
        f[7] = __builtin_amdgcn_alignbit(u3, u2, 23) & 0x1fff0u;
        uint4_t aop[8];
#pragma unroll
        for (int n = 0; n < 8; ++n)
          aop[n] = *reinterpret_cast<const uint4_t *>(reinterpret_cast<const char *>(sm.lut) + f[n]);
#pragma unroll
        for (int n = 0; n < 8; ++n)
          acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, aop[n]), pop[n * NACC / 8],
                                                          acc[n], 0, 0, 0);
      } else if constexpr (V3) {
        const uint2_t top = blk ? cur.vt1 : cur.vt0;
#define SKVQ_PV3(N, WORD, TOP)                                                                              \
  acc[N] = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack_v3_field<(N) & 3>(((N) & 1) ? (WORD) >> 8 : (WORD), TOP), \
                                                  pop[(N) * NACC / 8], acc[N], 0, 0, 0)
        SKVQ_PV3(0, raw.x, top.x); SKVQ_PV3(1, raw.x, top.x); SKVQ_PV3(2, raw.y, top.x); SKVQ_PV3(3, raw.y, top.x);
        SKVQ_PV3(4, raw.z, top.y); SKVQ_PV3(5, raw.z, top.y); SKVQ_PV3(6, raw.w, top.y); SKVQ_PV3(7, raw.w, top.y);
#undef SKVQ_PV3
      } else {
        const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int n = 0; n < 8; ++n) {
          const unsigned f = (n & 1) ? (w[n >> 1] >> 8) : w[n >> 1];
          acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack_v_field(f), pop[n * NACC / 8], acc[n], 0, 0, 0);
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
  };
  // Whole triples first.  The loop has no early exit: the wait counters the compiler places
  // are exact only if every path into the loop's top has the same loads in flight, in the
  // same order (buffer a's, then buffer b's).
  // (A 3- or 4-bit row or unit takes more registers, and unequal groups need an accumulator and a
  // weight operand per 16 positions: those variants rotate two buffers.)
  if constexpr (K4 || V4 || K3 || V3 || UNEQ) {
    while (tile_b < tile_end) {
      compute_tile(buf_a, tile_a);
      tile_a = tile_of(n_a += 2);
      buf_a = load_tile(min(tile_a, tile_cap));
      compute_tile(buf_b, tile_b);
      tile_b = tile_of(n_b += 2);
      buf_b = load_tile(min(tile_b, tile_cap));
    }
  } else {
  while (tile_c < tile_end) {
    buf_c = load_tile(min(tile_c, tile_cap));
    compute_tile(buf_a, tile_a);
    tile_a = tile_of(n_a += 3);
    buf_a = load_tile(min(tile_a, tile_cap));
    compute_tile(buf_b, tile_b);
    tile_b = tile_of(n_b += 3);
    buf_b = load_tile(min(tile_b, tile_cap));
    compute_tile(buf_c, tile_c);
    tile_c = tile_of(n_c += 3);
  }
  }
  // At most two tiles are left, already loaded into a and b.
#pragma unroll 1
  for (int k = 0; k < 2 && tile_a < tile_end; ++k) {
    compute_tile(buf_a, tile_a);
    buf_a = buf_b;
    tile_a = tile_b;
    tile_b = tile_end;
  }

  // ---- epilogue: fold lanes, columns, waves and ring slices; write this chunk's partial ----
  {
    // (all the sums first, then all the stores from lane 63: the chains of row moves interleave)
    float ls[R], zs[R][NG];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      ls[r] = wave_sum_in_last_lane(lsum[r]);
#pragma unroll
      for (int g = 0; g < NG; ++g) zs[r][g] = wave_sum_in_last_lane(zacc[r][g]);
    }
    if (lane == 63) {
#pragma unroll
      for (int r = 0; r < R; ++r) {
        sm.wm[r][wave] = first ? -INFINITY : mref[r];
        sm.wl[r][wave] = ls[r];
#pragma unroll
        for (int g = 0; g < NG; ++g) sm.wz[r][g][wave] = zs[r][g];
      }
    }
  }
  if (!first) {
    const int col = lane & 15, kb = lane >> 4;
    // codes carried 2^(4-24) (2-bit and 4-bit units) or 2^(8-24) (3-level units)
    const float unscale = (TERNARY ? 65536.0f : 1048576.0f) / beta;
#pragma unroll
    for (int n = 0; n < 8; ++n)
    {
      float4_t o4;
#pragma unroll
      for (int rr = 0; rr < 4; ++rr)
        o4[rr] = (acc[n][rr] + row_move<kRowShl + R>(acc[n][rr])) * unscale;  // + column R + r: the low halves' sum
      if (col < R) *reinterpret_cast<float4_t *>(&sm.wb[wave].stage[col][16 * n + 4 * kb]) = o4;
    }
  }
  __syncthreads();
  if (tid < R * kD && head0 + (tid >> 7) < n_rows) {
    // thread (head r, position p); a wavefront serves one head.  The sixteen things to combine --
    // the eight wavefronts' tile sums and their eight ring-slice sums -- are spread over the lanes of
    // every row of sixteen: lane i holds the reference and the weight sum of thing i, the chunk's
    // reference m* is a row maximum, thing i's factor 2^(m_i - m*) one exponential per lane instead
    // of sixteen per thread, the weight sum a row sum; the factors then reach every thread as
    // wave-uniform values read from lanes 0..15.
    const int r = tid >> 7, p = tid & 127;
    const int ch = pv_ch;
    static_assert(kNW == 8, "the epilogue spreads eight tile sums and eight ring sums over sixteen lanes");
    const int thing = lane & 15, src = thing & 7;
    const bool ring_thing = thing >= 8;
    float x = ring_thing ? sm.rm[r][src] : sm.wm[r][src];   // its reference
    const float y = ring_thing ? sm.rl[r][src] : sm.wl[r][src];  // its sum of weights
    const bool has_tokens = y > 0.f;  // (a wave or slice without tokens left no meaningful reference)
    x = has_tokens ? x : -INFINITY;
    float m = x;
    m = fmaxf(m, row_move<kQuadSwap1>(m));
    m = fmaxf(m, row_move<kQuadSwap2>(m));
    m = fmaxf(m, row_move<kRowHalfMirror>(m));
    m = fmaxf(m, row_move<kRowMirror>(m));  // every lane: the maximum of its row
    const float factor = has_tokens ? fast_exp2(x - m) : 0.f;
    float den = factor * y;
    den += row_move<kQuadSwap1>(den);
    den += row_move<kQuadSwap2>(den);
    den += row_move<kRowHalfMirror>(den);
    den += row_move<kRowMirror>(den);
    const int zg = UNEQ ? piece_group(p >> 4) : p * NG / kD;
    const float4_t z0 = *reinterpret_cast<const float4_t *>(&sm.wz[r][zg][0]);
    const float4_t z1 = *reinterpret_cast<const float4_t *>(&sm.wz[r][zg][4]);
    const float wz[kNW] = {z0[0], z0[1], z0[2], z0[3], z1[0], z1[1], z1[2], z1[3]};
    // (every read unconditional, what a wave or slice without tokens left there is deselected
    // afterwards: the reads then go out together and are waited for once, not one LDS round
    // trip after the other)
    float ws[kNW], rs[kNW];
#pragma unroll
    for (int w = 0; w < kNW; ++w) {
      ws[w] = sm.wb[w].stage[r][p] + wz[w];
      rs[w] = sm.ring_o[w][r][ch];
    }
    float num = 0.f;
#pragma unroll
    for (int w = 0; w < kNW; ++w) {
      const float e = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, factor), w));
      const float g = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, factor), 8 + w));
      num = fmaf(e, e > 0.f ? ws[w] : 0.f, num);
      num = fmaf(g, g > 0.f ? rs[w] : 0.f, num);
    }
    if (mo.mode == kMergeDirect) {
      // the only chunk of its kv head: this is the result
      const float o = num / den;
      const long long idx = row_index(head0 + r) * kD + ch;
      mo.out_f32[idx] = o;
      if (mo.out_f16) mo.out_f16[idx] = __float2half_rn(o);
    } else {
      float *part =
          L.workspace + (row_index(head0 + r) * (SKVQ_MAX_SPLITS + 1) + sp) * kPartialStride;
      part[4 + ch] = num;
      if (p == 0) {
        part[0] = m;
        part[1] = den;
      }
    }
  }
}

}  // namespace

// The launcher of the kernels with KL-level keys and VL-level values.
template <int KL, int VL>
hipError_t launch_decode_mfma_fmt(const Layout &L, const __half *q, long long T, long long nq, int n_sink,
                                  int n_splits, int n_new, const __half *knew, const __half *vnew, long long te,
                                  MergeOut mo, hipStream_t s) {
  if (T <= 0 || nq < 0 || nq > SKVQ_MAX_QUANT_TOKENS || T - nq > 0x7fffffff || n_splits < 1 ||
      n_splits > SKVQ_MAX_SPLITS)
    return hipErrorInvalidValue;
  if (n_new < 1 || n_new > SKVQ_MAX_NEW_TOKENS || L.R > 8) return hipErrorInvalidValue;
  const int n_rows = n_new * L.R;
  const int passes = decode_passes(n_rows), rk = n_rows == 1 ? 1 : n_rows == 2 ? 2 : 4;
  if ((knew != nullptr) != (vnew != nullptr) || (knew && (passes != 1 || n_new != 1))) return hipErrorInvalidValue;
  if (knew && T - 1 >= L.W && (te < 0 || te >= L.Tcap || te != nq - 1)) return hipErrorInvalidValue;
  if ((long long)L.Hk * passes > 65535) return hipErrorInvalidValue;
  if (mo.mode != kMergeSeparate && !mo.out_f32) return hipErrorInvalidValue;
  if (mo.mode == kMergeDirect && n_splits != 1) return hipErrorInvalidValue;
  const dim3 grid(n_splits, L.Hk * passes, L.B), block(kThreads);
  const ChunkPlan plan = plan_chunks(L, T, nq, n_sink, n_splits, knew != nullptr);
#define SKVQ_LAUNCH(RR, MM, GG, UU) \
  hipLaunchKernelGGL((decode_mfma_kernel<RR, KL, VL, MM, GG, UU>), grid, block, 0, s, L, q, T, nq, n_sink, n_splits, passes, n_new, knew, vnew, te, plan, mo)
#define SKVQ_LAUNCH_NG(RR, MM)                                                                   \
  switch (L.NG) {                                                                                \
    case 1: SKVQ_LAUNCH(RR, MM, 1, false); break;                                                \
    case 2: if (L.uneq) SKVQ_LAUNCH(RR, MM, 2, true); else SKVQ_LAUNCH(RR, MM, 2, false); break; \
    case 4: if (L.uneq) SKVQ_LAUNCH(RR, MM, 4, true); else SKVQ_LAUNCH(RR, MM, 4, false); break; \
    default: return hipErrorInvalidValue;                                                        \
  }
#define SKVQ_LAUNCH_META(RR)                                                \
  switch (L.meta_fmt) {                                                     \
    case SKVQ_META_F32: SKVQ_LAUNCH_NG(RR, SKVQ_META_F32) break;            \
    case SKVQ_META_F16: SKVQ_LAUNCH_NG(RR, SKVQ_META_F16) break;            \
    case SKVQ_META_FP8_E4M3: SKVQ_LAUNCH_NG(RR, SKVQ_META_FP8_E4M3) break;  \
    default: return hipErrorInvalidValue;                                   \
  }
  if (L.k_levels != KL || L.v_levels != VL) return hipErrorInvalidValue;
  switch (rk) {
    case 1: SKVQ_LAUNCH_META(1) break;
    case 2: SKVQ_LAUNCH_META(2) break;
    case 4: SKVQ_LAUNCH_META(4) break;
    default: return hipErrorInvalidValue;
  }
#undef SKVQ_LAUNCH_META
#undef SKVQ_LAUNCH_NG
#undef SKVQ_LAUNCH
  return hipGetLastError();
}

}  // namespace skvq
