// Matrix-core chunk kernel of skvq_decode_attention for gfx950 (group size 128, up to four
// query heads per kv head).
//
// Per wavefront, per tile of 64 packed tokens:
//   QK   S^T[head][token] by 32 v_mfma_f32_4x4x4_16b_f16 (16 independent 4x4 blocks, lane =
//        token): the B operand is the lane's own 32-byte key row, its 2-bit codes turned into
//        fp16 SUBNORMALS by one AND each (a code c sitting at mantissa bit s is the fp16 value
//        c*2^(s-24)); the A operand is the reordered query, pre-multiplied by the matching
//        power of two, held in registers.  Afterwards lane l holds the scores of token l for
//        the (up to) four heads.
//   softmax  lazily re-referenced online softmax in the exp2 domain: the running reference m
//        only moves when a score exceeds it by more than 2^6 (wave-uniform branch).
//   PV   O^T[channel][head] by 16 v_mfma_f32_16x16x32_f16: the A operand is the V block unit
//        that the lane loaded (8 tokens x 8 channels, token-minor; 3-level units go through a
//        13-bit -> 8-code table in LDS), the B operand holds p*scale split into a high and a
//        low fp16 part (two columns per head) so that the weights keep ~22 bits.
// The zero-points never enter the matrix products: sum_p q_p (s c_p + z) = s sum q c + z sum q
// and sum_t w_t (s_t c + z_t) = sum (w_t s_t) c + sum w_t z_t.
//
// The matrix core accumulates products of subnormal inputs as if their mantissa were full, so
// a code at mantissa bit s costs about (10 - s) bits of the accumulator's precision; every
// code is therefore moved to bit 4, 6 or 8 before it is masked out.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <math.h>

#include "skvq_internal.h"

namespace skvq {
#ifdef SKVQ_TIMING
__device__ unsigned long long skvq_timing[8 * 4096];
#define SKVQ_STAMP(slot)                                                                    \
  if (threadIdx.x == 0)                                                                     \
  skvq_timing[8 * ((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) + (slot)] = \
      __builtin_amdgcn_s_memrealtime()
#else
#define SKVQ_STAMP(slot)
#endif
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
constexpr float kRefSlack = 6.0f;    // scores may exceed the running reference by 2^6
constexpr float kVsTarget = 256.0f;  // max(v scale)*beta is brought below this ...
constexpr float kVsLimit = 512.0f;   // ... and re-normalised when a token exceeds this
constexpr unsigned kM4 = 0x00300030u, kM6 = 0x00c000c0u, kM8 = 0x03000300u;

__device__ __forceinline__ float wave_max(float v) {
  for (int off = 32; off; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  for (int off = 32; off; off >>= 1) v += __shfl_xor(v, off);
  return v;
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

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
  union {
    unsigned lut[TERNARY ? 8192 : 1];  // main loop: 13-bit field -> eight codes
    float stage[4][2 * R][kD];         // epilogue: O^T per wave and column
  };
  float qraw[4][kD];                   // the query heads as loaded (rows >= R are zero)
  _Float16 qa[32][4][4];               // A operands of the score product: [step][head][k slot]
  float qsum[4];                       // sm_scale*log2(e) * sum of the query, per head
  float qinit[4];                      // -1.5 * sum of the query, in the score product's units (2^-16)
  _Float16 pbuf[4][2][2 * R][32];      // per wave: [block][column][token slot]
  float wm[4][R], wl[4][R], wz[4][R];
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

// ---------------------------------------------------------------------------------------
// The fp16 ring (last W tokens, original channel order) as one more chunk, in tiles of 64
// tokens staged through LDS: plain vector arithmetic.  Scores: four threads per token, 32
// channels each.  Value sum: thread = (channel pair, quarter of the tile).  The next tile's
// rows are already in flight while a tile is computed.
// ---------------------------------------------------------------------------------------
constexpr int kRingTile = 64;
constexpr int kRingKStride = kD + 8;  // halves; the padding spreads the rows over the LDS banks

template <int R>
struct RingSmem {
  __half kt[kRingTile][kRingKStride];
  __half vt[kRingTile][kD];
  float qf[R][kD];          // query * sm_scale * log2(e)
  float sc[R][kRingTile];   // scores, then softmax numerators, of the current tile
  float m[R], l[R], scale[R];
  float accs[4][R][kD];
};

template <int R>
__device__ void ring_chunk(const Layout &L, RingSmem<R> &rs, const __half *__restrict__ q, long long T,
                           long long nq, int part_index) {
  // This workgroup is short and latency-bound; let its waves win the issue arbitration against
  // the packed chunks they share the compute unit with, so that it is never the last to end.
  __builtin_amdgcn_s_setprio(3);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int hk = blockIdx.y, b = blockIdx.z;
  const long long head = (long long)b * L.Hk + hk;
  const float c = L.sm_scale * kLog2e;
  const int n_win = (int)(T - nq), W = L.W;
  const uint4_t *kwin = reinterpret_cast<const uint4_t *>(L.k_win + head * W * kD);
  const uint4_t *vwin = reinterpret_cast<const uint4_t *>(L.v_win + head * W * kD);
  const int tk = tid >> 2, qt = tid & 3;   // scores: token of the tile, quarter of its channels
  const int cp = tid & 63, tq = tid >> 6;  // values: channel pair, quarter of the tile
  const int slot0 = (int)(nq % W);         // ring slot of the first ring token

  // staging: thread copies 16-byte piece (tid%16) of rows tid/16 + 16*i, i = 0..3, of K and of V
  const int crow = tid >> 4, cpiece = tid & 15;
  uint4_t kst[4], vst[4];
  auto load_stage = [&](int tile0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int t = tile0 + crow + 16 * i;
      if (t >= n_win) t = n_win - 1;  // rows past the end repeat the last one; they get weight 0
      int slot = slot0 + t;
      slot -= (slot / W) * W;
      kst[i] = kwin[(size_t)slot * 16 + cpiece];
      vst[i] = vwin[(size_t)slot * 16 + cpiece];
    }
  };
  load_stage(0);
  for (int x = tid; x < R * kD; x += 256)
    rs.qf[x >> 7][x & 127] = c * __half2float(q[((long long)b * L.Hq + hk * R + (x >> 7)) * kD + (x & 127)]);
  if (tid < R) rs.m[tid] = -INFINITY, rs.l[tid] = 0.f;

  float acc[R][2];
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r][0] = acc[r][1] = 0.f;

  for (int tile0 = 0; tile0 < n_win; tile0 += kRingTile) {
    const int n_in = n_win - tile0 < kRingTile ? n_win - tile0 : kRingTile;
    __syncthreads();  // the previous tile's kt/vt/sc are no longer read
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      *reinterpret_cast<uint4_t *>(&rs.kt[crow + 16 * i][8 * cpiece]) = kst[i];
      *reinterpret_cast<uint4_t *>(&rs.vt[crow + 16 * i][8 * cpiece]) = vst[i];
    }
    if (tile0 + kRingTile < n_win) load_stage(tile0 + kRingTile);
    __syncthreads();

    // ---- scores: 32 channels per thread ----
    float s[R];
#pragma unroll
    for (int r = 0; r < R; ++r) s[r] = 0.f;
#pragma unroll 1
    for (int i = 0; i < 4; ++i) {
      const half8_t x = *reinterpret_cast<const half8_t *>(&rs.kt[tk][32 * qt + 8 * i]);
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const float4_t qa = *reinterpret_cast<const float4_t *>(&rs.qf[r][32 * qt + 8 * i]);
        const float4_t qb = *reinterpret_cast<const float4_t *>(&rs.qf[r][32 * qt + 8 * i + 4]);
        s[r] = fmaf(qa[0], (float)x[0], s[r]);
        s[r] = fmaf(qa[1], (float)x[1], s[r]);
        s[r] = fmaf(qa[2], (float)x[2], s[r]);
        s[r] = fmaf(qa[3], (float)x[3], s[r]);
        s[r] = fmaf(qb[0], (float)x[4], s[r]);
        s[r] = fmaf(qb[1], (float)x[5], s[r]);
        s[r] = fmaf(qb[2], (float)x[6], s[r]);
        s[r] = fmaf(qb[3], (float)x[7], s[r]);
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      s[r] += __shfl_xor(s[r], 1);
      s[r] += __shfl_xor(s[r], 2);
      if (qt == 0) rs.sc[r][tk] = tk < n_in ? s[r] : -INFINITY;
    }
    __syncthreads();
    for (int r = wave; r < R; r += 4) {  // one wavefront per head: tile max, numerators, sum
      const float v0 = rs.sc[r][lane];
      const float tm = wave_max(v0);
      const float mold = rs.m[r], mnew = fmaxf(mold, tm);
      const float p0 = exp2f(v0 - mnew);  // -inf gives 0
      rs.sc[r][lane] = p0;
      const float sum = wave_sum(p0);
      if (lane == 0) {
        const float sc_old = exp2f(mold - mnew);  // 0 on the first tile
        rs.m[r] = mnew;
        rs.scale[r] = sc_old;
        rs.l[r] = rs.l[r] * sc_old + sum;
      }
    }
    __syncthreads();
    // ---- values: 16 tokens per thread ----
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r][0] *= rs.scale[r], acc[r][1] *= rs.scale[r];
#pragma unroll 4
    for (int k = 0; k < 16; ++k) {
      const __half2 v2 = *reinterpret_cast<const __half2 *>(&rs.vt[16 * tq + k][2 * cp]);
      const float vx = __low2float(v2), vy = __high2float(v2);
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const float p = rs.sc[r][16 * tq + k];  // 0 for tokens past the end
        acc[r][0] = fmaf(p, vx, acc[r][0]);
        acc[r][1] = fmaf(p, vy, acc[r][1]);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r) rs.accs[tq][r][2 * cp] = acc[r][0], rs.accs[tq][r][2 * cp + 1] = acc[r][1];
  __syncthreads();
  for (int x = tid; x < R * kD; x += 256) {
    const int r = x >> 7, ch = x & 127;
    float *part = L.workspace + (((long long)b * L.Hq + hk * R + r) * (SKVQ_MAX_SPLITS + 1) + part_index) * kPartialStride;
    part[4 + ch] = rs.accs[0][r][ch] + rs.accs[1][r][ch] + rs.accs[2][r][ch] + rs.accs[3][r][ch];
    if (ch == 0) {
      part[0] = rs.m[r];
      part[1] = rs.l[r];
    }
  }
}

// What one wavefront loads for one tile of 64 tokens.
struct TileData {
  uint4_t k0, k1;       // lane = token: its 32-byte key row
  float2 kmeta, vmeta;  // lane = token: (scale, zero)
  Unit16 v0, v1;        // lane = unit of V block 2*tile and 2*tile+1
};

template <int R, bool TERNARY>
__global__ __launch_bounds__(256, 3) void decode_mfma_kernel(Layout L, const __half *__restrict__ q,
                                                             long long T, long long nq, int n_splits,
                                                             int tiles_per_split) {
  // grid (n_splits + 1, Hk, B): x = 0 is the fp16 ring (partial index n_splits), x = 1 + sp
  // is packed chunk sp.  The ring goes first so that it runs beside the packed chunks.
  __shared__ union SharedUnion {
    Smem<R, TERNARY> sm;
    RingSmem<R> rs;
    __device__ SharedUnion() {}
  } shared;
  SKVQ_STAMP(0);
  if (blockIdx.x == 0) {
    ring_chunk<R>(L, shared.rs, q, T, nq, n_splits);
    SKVQ_STAMP(3);
    return;
  }
  Smem<R, TERNARY> &sm = shared.sm;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int sp = blockIdx.x - 1, hk = blockIdx.y, b = blockIdx.z;
  const long long head = (long long)b * L.Hk + hk;
  const float c = L.sm_scale * kLog2e;

  // ---- this chunk, this wave's tiles ----
  const int n_tiles = (int)((nq + 63) >> 6);
  (void)tiles_per_split;  // the packed tiles are dealt out evenly: chunk sizes differ by at most one
  const int tile_begin = (int)(((long long)sp * n_tiles) / n_splits);
  const int tile_end = (int)(((long long)(sp + 1) * n_tiles) / n_splits);

  const uint8_t *kc = L.k_codes + head * L.Tcap * (kD / 4);
  const float2 *km = reinterpret_cast<const float2 *>(L.k_meta) + head * L.Tcap;
  const float2 *vm = reinterpret_cast<const float2 *>(L.v_meta) + head * L.Tcap;
  const uint8_t *vc = L.v_codes + head * L.n_vblocks * L.v_block_bytes;
  const int last_blk = (int)((nq - 1) >> 5);
  const int vbb = TERNARY ? kTernaryBlockBytes : kTwoBitBlockBytes;
  const unsigned unit_off = TERNARY ? ((13 * lane) & ~3) : 16 * lane;
  const int unit_sh = TERNARY ? ((13 * lane) & 3) : 0;
  // token slot i = lane%8 sits in register m = i/2 at bit {4,6,8,8}[m]: undo 2^(bit-4)
  const float kslot_scale = ((lane >> 1) & 3) == 0 ? 1.f : ((lane >> 1) & 3) == 1 ? 0.25f : 0.0625f;
  const int last_token = (int)(nq - 1);

  auto load_tile = [&](int tile) {
    TileData d;
    int t = tile * 64 + lane;
    if (t > last_token) t = last_token;  // only in the last tile; such lanes are masked below
    const uint4_t *krow = reinterpret_cast<const uint4_t *>(kc + (size_t)tile * 2048) + 2 * lane;
    if (tile * 64 + 63 > last_token) krow = reinterpret_cast<const uint4_t *>(kc + (size_t)t * 32);
    d.k0 = krow[0];
    d.k1 = krow[1];
    d.kmeta = km[t];
    d.vmeta = vm[t];
    const int blk0 = 2 * tile;
    const int blk1 = blk0 + 1 > last_blk ? last_blk : blk0 + 1;
    d.v0 = *reinterpret_cast<const Unit16 *>(vc + (size_t)blk0 * vbb + unit_off);
    d.v1 = *reinterpret_cast<const Unit16 *>(vc + (size_t)blk1 * vbb + unit_off);
    return d;
  };

  // ---- prologue: one memory round trip (first tile, table, query, permutation), then LDS ----
  int tile = tile_begin + wave;
  TileData cur, nxt;
  if (tile < tile_end) cur = load_tile(tile);
  nxt = cur;
  if (tile + 4 < tile_end) nxt = load_tile(tile + 4);
  {
    const int r = tid >> 6;  // 64 threads load one query head as half2
    __half2 q2 = __floats2half2_rn(0.f, 0.f);
    if (r < R) q2 = reinterpret_cast<const __half2 *>(q + ((long long)b * L.Hq + hk * R + r) * kD)[lane];
    const int pk = L.perm_k[hk * kD + (tid & 127)];
    if (TERNARY) {
      const uint4_t *src = reinterpret_cast<const uint4_t *>(L.trit_lut);
      uint4_t *dst = reinterpret_cast<uint4_t *>(sm.lut);
#pragma unroll
      for (int x = 0; x < 7; ++x)  // 6561 entries = 1641 16-byte pieces; fields of valid data stay below
        if (tid + 256 * x < 1641) dst[tid + 256 * x] = src[tid + 256 * x];
    }
    sm.qraw[r][2 * lane] = __low2float(q2);
    sm.qraw[r][2 * lane + 1] = __high2float(q2);
    __syncthreads();
#pragma unroll
    for (int rr = 0; rr < 2; ++rr) {  // thread (p = tid%128, heads tid/128 and tid/128 + 2)
      const int row = (tid >> 7) + 2 * rr, p = tid & 127;
      int step, kslot, shift;
      k_slot_of(p, step, kslot, shift);
      sm.qa[step][row][kslot] = (_Float16)ldexpf(sm.qraw[row][pk], 8 - shift);  // exact: a power of two
    }
    const float v = wave_sum(sm.qraw[wave][lane] + sm.qraw[wave][lane + 64]);  // wave r sums head r
    if (lane == 0) {
      sm.qsum[wave] = c * v;
      sm.qinit[wave] = -1.5f * v * (1.0f / 65536.0f);
    }
    __syncthreads();
  }
  // lane l supplies row l%4 (= head) of step l/4 (first register pair) and 16 + l/4 (second)
  const half4_t qop_lo = *reinterpret_cast<const half4_t *>(sm.qa[lane >> 2][lane & 3]);
  const half4_t qop_hi = *reinterpret_cast<const half4_t *>(sm.qa[16 + (lane >> 2)][lane & 3]);
  float qsc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) qsc[r] = sm.qsum[r];
  // The score accumulators start at -1.5*sum(q): the products then sum q*(c - 1.5), centred
  // codes, which keeps both halves of  scale*sum q(c-1.5) + (zero+1.5 scale)*sum q  small.
  const float4_t dinit = {sm.qinit[0], sm.qinit[1], sm.qinit[2], sm.qinit[3]};

  float mref[R], lsum[R], zacc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) mref[r] = 0.f, lsum[r] = 0.f, zacc[r] = 0.f;
  float beta = 1.f;
  float4_t acc[8];
#pragma unroll
  for (int n = 0; n < 8; ++n) acc[n] = float4_t{0.f, 0.f, 0.f, 0.f};
  bool first = true;

  SKVQ_STAMP(1);
  for (; tile < tile_end; tile += 4) {
    TileData nxt2 = nxt;
    if (tile + 8 < tile_end) nxt2 = load_tile(tile + 8);  // two tiles are in flight while this one is computed
    const bool valid = tile * 64 + lane <= last_token;

    // ---- scores: 32 products of 4 channels each ----
    float4_t d0 = dinit;
    d0 = qk_dword<0>(cur.k0.x, qop_lo, qop_hi, d0);
    d0 = qk_dword<1>(cur.k0.y, qop_lo, qop_hi, d0);
    d0 = qk_dword<2>(cur.k0.z, qop_lo, qop_hi, d0);
    d0 = qk_dword<3>(cur.k0.w, qop_lo, qop_hi, d0);
    d0 = qk_dword<4>(cur.k1.x, qop_lo, qop_hi, d0);
    d0 = qk_dword<5>(cur.k1.y, qop_lo, qop_hi, d0);
    d0 = qk_dword<6>(cur.k1.z, qop_lo, qop_hi, d0);
    d0 = qk_dword<7>(cur.k1.w, qop_lo, qop_hi, d0);
    // u = log2-domain score minus the running reference
    const float a_t = cur.kmeta.x * (c * 65536.0f);       // codes carry 2^(s-24), the query 2^(8-s)
    const float zc = fmaf(1.5f, cur.kmeta.x, cur.kmeta.y);  // dequantized value of the centre code 1.5
    float u[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      u[r] = fmaf(d0[r], a_t, fmaf(zc, qsc[r], -mref[r]));
      if (!valid) u[r] = -INFINITY;
    }
    const float vs = valid ? cur.vmeta.x : 0.f;
    const float vz = valid ? cur.vmeta.y : 0.f;
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
          (void)frexpf(vsmax, &e);  // vsmax = fr * 2^e, fr in [0.5, 1)
          nb = ldexpf(1.f, 8 - e);  // vsmax * nb in [128, 256)
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

    // ---- weights: p = 2^u, P' = p * vscale * beta * 2^-(bit-4), split into high and low fp16 ----
    const float vsb = vs * beta * kslot_scale;
    _Float16 *pw = &sm.pbuf[wave][lane >> 5][0][lane & 31];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float p = fast_exp2(u[r]);
      lsum[r] += p;
      zacc[r] = fmaf(p, vz, zacc[r]);
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
      const Unit16 raw = blk ? cur.v1 : cur.v0;
      if (TERNARY) {
        const unsigned u0 = __builtin_amdgcn_alignbyte(raw.y, raw.x, unit_sh);
        const unsigned u1 = __builtin_amdgcn_alignbyte(raw.z, raw.y, unit_sh);
        const unsigned u2 = __builtin_amdgcn_alignbyte(raw.w, raw.z, unit_sh);
        const unsigned u3 = raw.w >> (8 * unit_sh);
        unsigned f[8], fld[8];
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
    cur = nxt;
    nxt = nxt2;
  }

  SKVQ_STAMP(2);
  // ---- epilogue: fold columns, lanes and the four waves; write this chunk's partial ----
  __syncthreads();  // `stage` shares its memory with the table that slower waves may still read
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
    const float mstar = fmaxf(fmaxf(sm.wm[0][r], sm.wm[1][r]), fmaxf(sm.wm[2][r], sm.wm[3][r]));
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
  SKVQ_STAMP(3);
}

}  // namespace

#ifdef SKVQ_TIMING
extern "C" int skvq_debug_read_timing(unsigned long long *host, int n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(skvq_timing), sizeof(unsigned long long) * n);
}
#endif

bool decode_mfma_supported(const Layout &L) { return L.G == kD && (L.R == 1 || L.R == 2 || L.R == 4); }

hipError_t launch_decode_mfma(const Layout &L, const __half *q, long long T, long long nq, int n_splits,
                              long long tiles_per_split, hipStream_t s) {
  if (nq <= 0 || nq > 0x7fffffffll * 32 || tiles_per_split > 0x7fffffff || T - nq > 0x7fffffff)
    return hipErrorInvalidValue;
  const dim3 grid(n_splits + 1, L.Hk, L.B), block(256);
  const int tps = (int)tiles_per_split;
#define SKVQ_LAUNCH(RR, TT) \
  hipLaunchKernelGGL((decode_mfma_kernel<RR, TT>), grid, block, 0, s, L, q, T, nq, n_splits, tps)
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
