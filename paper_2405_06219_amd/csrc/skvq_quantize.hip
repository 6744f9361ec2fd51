// Quantize-on-evict and prefill-quantize kernels (Section 3.1 Eq. 2, Section 3.2,
// Algorithm 1 clipping_quant) for gfx950.
//
// Append: one wavefront owns one (token, kv head) row; lane l holds the two reordered
// positions 2l and 2l+1 and the group minimum/maximum is a cross-lane butterfly over the G/2
// lanes of a group.  Prefill: one wavefront owns eight rows; a lane holds sixteen consecutive
// reordered positions of one of them.  Every fp32 operation of Eq. 2 is issued as an explicitly
// rounded intrinsic so that the compiler can neither fuse nor reorder them.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include "skvq_internal.h"
#include "skvq_meta.h"

namespace skvq {
namespace {

// Eq. 2 parameters of one group from its min and max.
struct GroupParams {
  float lo, scale, inv;
  unsigned stored;  // storage word of (scale, lo) in the compact formats
};

__device__ __forceinline__ GroupParams group_params(float mn, float mx, float alpha, float top, int fmt) {
  if (mn == 0.0f) mn = 0.0f;  // a minimum of -0 is stored as +0
  if (mx == 0.0f) mx = 0.0f;
  GroupParams g;
  const float lo = __fmul_rn(alpha, mn);
  const float hi = __fmul_rn(alpha, mx);
  // the codes are computed with the values that decoding will read back from storage
  const MetaPair m = meta_make(__fdiv_rn(__fsub_rn(hi, lo), top), lo, fmt);
  g.lo = m.zero;
  g.scale = m.scale;
  g.stored = m.stored;
  g.inv = g.scale > 0.0f ? __fdiv_rn(1.0f, g.scale) : 0.0f;
  return g;
}

__device__ __forceinline__ unsigned encode(float x, const GroupParams &g, float top) {
  float r = rintf(__fmul_rn(__fsub_rn(x, g.lo), g.inv));
  r = r < 0.0f ? 0.0f : r;
  r = r > top ? top : r;
  return (unsigned)r;
}

// Group of the 16 positions 16n .. 16n+15 (Layout::gmap).
__device__ __forceinline__ int tile_group(unsigned gmap, int n) { return (gmap >> (4 * n)) & 15; }

// min and max over the G/2 consecutive lanes that hold one group (lane l: positions 2l, 2l+1)
__device__ __forceinline__ void group_minmax(float &mn, float &mx, int G) {
  for (int off = 1; off < G / 2; off <<= 1) {
    mn = fminf(mn, __shfl_xor(mn, off));
    mx = fmaxf(mx, __shfl_xor(mx, off));
  }
}
// The same for unequal groups (whole 16-position tiles, 8 lanes each): first over the lanes of a
// tile, then over the other seven tiles, taking those of the lane's own group.
__device__ __forceinline__ void group_minmax_unequal(float &mn, float &mx, int lane, unsigned gmap) {
  for (int off = 1; off < 8; off <<= 1) {
    mn = fminf(mn, __shfl_xor(mn, off));
    mx = fmaxf(mx, __shfl_xor(mx, off));
  }
  const int tile = lane >> 3, g = tile_group(gmap, tile);
  const float tmn = mn, tmx = mx;
#pragma unroll
  for (int k = 1; k < 8; ++k) {
    const int other = (tile + k) & 7;
    const float omn = __shfl(tmn, 8 * other + (lane & 7)), omx = __shfl(tmx, 8 * other + (lane & 7));
    if (tile_group(gmap, other) == g) {
      mn = fminf(mn, omn);
      mx = fmaxf(mx, omx);
    }
  }
}

// Reorder one row through LDS and encode it.  row_lds: 128 halves of this wavefront.
// Returns this lane's two codes and the group's (scale, zero).
__device__ __forceinline__ void encode_row(const __half *row_lds, int p0, int p1, float alpha, int G,
                                           float top, int fmt, bool uneq, unsigned gmap, int lane, unsigned &c0,
                                           unsigned &c1, MetaPair &meta) {
  const float x0 = __half2float(row_lds[p0]);
  const float x1 = __half2float(row_lds[p1]);
  float mn = fminf(x0, x1), mx = fmaxf(x0, x1);
  if (uneq)
    group_minmax_unequal(mn, mx, lane, gmap);
  else
    group_minmax(mn, mx, G);
  const GroupParams g = group_params(mn, mx, alpha, top, fmt);
  c0 = encode(x0, g, top);
  c1 = encode(x1, g, top);
  meta = MetaPair{g.scale, g.lo, g.stored};
}

// K row: position p at bits [2p, 2p+2).  Lane l contributes 4 bits; 8 lanes form a dword.
__device__ __forceinline__ void store_k_row(uint8_t *row, int lane, unsigned c0, unsigned c1) {
  unsigned w = (c0 | (c1 << 2)) << (4 * (lane & 7));
  w |= __shfl_xor(w, 1);
  w |= __shfl_xor(w, 2);
  w |= __shfl_xor(w, 4);
  if ((lane & 7) == 0) reinterpret_cast<unsigned *>(row)[lane >> 3] = w;
}

// 4-bit K row: position p at bits [4p, 4p+4).  Lane l contributes one byte; 4 lanes form a dword.
__device__ __forceinline__ void store_k_row4(uint8_t *row, int lane, unsigned c0, unsigned c1) {
  unsigned w = (c0 | (c1 << 4)) << (8 * (lane & 3));
  w |= __shfl_xor(w, 1);
  w |= __shfl_xor(w, 2);
  if ((lane & 3) == 0) reinterpret_cast<unsigned *>(row)[lane >> 2] = w;
}

// 3-bit formats: a 2-bit plane (laid out as the 2-bit format) plus a plane of top bits.  Top bit
// of the key at position p: dword p/32 of the plane, bit 16*((p%16)/8) + kKsig[(p%32)/16][p%8];
// of value code (n, i): dword n/4 of the unit's plane, bit 16*(i%2) + vtau(n%4, i/2).  The tables,
// one nibble per entry:
constexpr unsigned kKsig0 = 0x58643120u, kKsig1 = 0xefdbca97u;
__device__ __forceinline__ int ksig(int d, int e) { return ((d ? kKsig1 : kKsig0) >> (4 * e)) & 15; }
__device__ __forceinline__ int vtau(int nn, int m) { return m < 3 ? (nn & 1) + 6 * (nn >> 1) + 2 * m : 12 + nn; }

// Sixteen top bits of one key dword (position e at bit e) -> their places in the plane dword
// (d = 0: the even key dword of the pair, d = 1: the odd one).
__device__ __forceinline__ unsigned place_key_top_bits(unsigned y, int d) {
  const unsigned x = (y & 0xffu) | ((y & 0xff00u) << 8);  // e = 0..7 at bits 0..7, e = 8..15 at bits 16..23
  // d = 0: positions e -> {0,2,1,3,4,6,8,5}
  const unsigned a = (x & 0x00190019u) | ((x & 0x00220022u) << 1) | ((x & 0x00040004u) >> 1) |
                     ((x & 0x00400040u) << 2) | ((x & 0x00800080u) >> 2);
  // d = 1: positions e -> {7,9,10,12,11,13,15,14}
  const unsigned b = ((x & 0x00910091u) << 7) | ((x & 0x00260026u) << 8) | ((x & 0x00480048u) << 9);
  return d ? b : a;
}

// 3-bit K row from the append kernel's lanes (lane l: positions 2l, 2l+1): the 2-bit plane as
// store_k_row, then the top-bit plane (16 lanes form a dword).
__device__ __forceinline__ void store_k_row3(uint8_t *row, int lane, unsigned c0, unsigned c1) {
  unsigned w = ((c0 & 3u) | ((c1 & 3u) << 2)) << (4 * (lane & 7));
  w |= __shfl_xor(w, 1);
  w |= __shfl_xor(w, 2);
  w |= __shfl_xor(w, 4);
  if ((lane & 7) == 0) reinterpret_cast<unsigned *>(row)[lane >> 3] = w;
  const int p = 2 * lane, d = (p >> 4) & 1, half = (p >> 3) & 1;
  unsigned h = ((c0 >> 2) << (16 * half + ksig(d, p & 7))) | ((c1 >> 2) << (16 * half + ksig(d, (p & 7) + 1)));
  h |= __shfl_xor(h, 1);
  h |= __shfl_xor(h, 2);
  h |= __shfl_xor(h, 4);
  h |= __shfl_xor(h, 8);
  if ((lane & 15) == 0) reinterpret_cast<unsigned *>(row + 32)[lane >> 4] = h;
}

// Spread eight 2-bit codes (token i at bits [2i,2i+2)) to the V unit order: token i goes to
// bit 16*(i%2) + 2*(i/2).
__device__ __forceinline__ unsigned spread_tokens(unsigned c8) {
  unsigned r = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) r |= ((c8 >> (2 * i)) & 3u) << (16 * (i & 1) + 2 * (i >> 1));
  return r;
}

// Base-3 number of eight codes (token i is digit i).
__device__ __forceinline__ unsigned trit_field(unsigned c8) {
  unsigned f = 0, pw = 1;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    f += ((c8 >> (2 * i)) & 3u) * pw;
    pw *= 3;
  }
  return f;
}

// ---------------------------------------------------------------------------------------
// Prefill: one workgroup (4 wavefronts) per V block of 32 tokens of one (b, hk); wavefront w
// handles the 8 tokens of sub-block kb = w, K and V, and builds that sub-block's 16 V units.
//
// The 8 fp16 rows of a wavefront (2 KB, contiguous in the source) arrive with two 16-byte loads
// per lane and are parked in LDS.  Lane (i = lane / 8, n = lane % 8) then owns the 16 reordered
// positions 16n .. 16n+15 of token i: it gathers them through the permutation, reduces
// min/max with the other lanes of its group, and encodes them (Eq. 2).  Its sixteen key codes
// are dword n of the token's packed row, so a wavefront stores 256 contiguous bytes.  Its
// sixteen value codes are exactly the codes (n, i) of units j = 0..15, which a second set of
// lanes (j = lane % 16, two fields each) collects from LDS to build the units.
// ---------------------------------------------------------------------------------------
constexpr int kRowStride = 136;  // halves per parked row: 272 B keeps 16-byte alignment and
                                 // puts the same channel of the 8 rows in 8 different banks

// Gathers positions 16n..16n+15 of one parked row, finds the group's Eq. 2 parameters and
// returns this lane's 16 codes.  BITS = 2: two bits each in .x (position 16n + e at bits [2e, 2e+2));
// BITS = 3: the low two bits like that in .x and the top bits in .y (position e at bit e);
// BITS = 4: four bits each in .x (e = 0..7 at bits [4e, 4e+4)) and .y (e = 8..15).
template <int BITS>
__device__ __forceinline__ uint2 encode16(const __half *row, const int4 (&pm)[4], float alpha, int G,
                                          float top, int fmt, bool uneq, unsigned gmap, int lane,
                                          GroupParams &gp) {
  const int ch[16] = {pm[0].x, pm[0].y, pm[0].z, pm[0].w, pm[1].x, pm[1].y, pm[1].z, pm[1].w,
                      pm[2].x, pm[2].y, pm[2].z, pm[2].w, pm[3].x, pm[3].y, pm[3].z, pm[3].w};
  float x[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) x[e] = __half2float(row[ch[e]]);
  float mn = x[0], mx = x[0];
#pragma unroll
  for (int e = 1; e < 16; ++e) {
    mn = fminf(mn, x[e]);
    mx = fmaxf(mx, x[e]);
  }
  if (uneq) {
    // unequal groups: the other seven 16-position pieces of the token sit in the other seven lanes
    // of this lane's group of eight; take those that belong to the same group
    const int n = lane & 7, g = tile_group(gmap, n);
    const float tmn = mn, tmx = mx;
#pragma unroll
    for (int k = 1; k < 8; ++k) {
      const int other = (n + k) & 7;
      const float omn = __shfl(tmn, (lane & ~7) + other), omx = __shfl(tmx, (lane & ~7) + other);
      if (tile_group(gmap, other) == g) {
        mn = fminf(mn, omn);
        mx = fmaxf(mx, omx);
      }
    }
  } else {
    for (int off = 1; off < G / 16; off <<= 1) {
      mn = fminf(mn, __shfl_xor(mn, off));
      mx = fmaxf(mx, __shfl_xor(mx, off));
    }
  }
  gp = group_params(mn, mx, alpha, top, fmt);
  // code = rint(clamp(y, 0, top)): clamping first gives the same integer because the bounds are
  // integers; adding 1.5 * 2^23 rounds to the nearest integer, ties to even, and leaves the code
  // in the low bits of the sum, which alignbit shifts into the row word from the top.
  unsigned w0 = 0, w1 = 0;
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const float y = __fmul_rn(__fsub_rn(x[e], gp.lo), gp.inv);
    const float r = __fadd_rn(__builtin_amdgcn_fmed3f(y, 0.0f, top), 12582912.0f);
    if (BITS == 2) {
      w0 = __builtin_amdgcn_alignbit(__float_as_uint(r), w0, 2);
    } else if (BITS == 3) {
      w0 = __builtin_amdgcn_alignbit(__float_as_uint(r), w0, 2);
      w1 = __builtin_amdgcn_alignbit(__float_as_uint(r) >> 2, w1, 1);
    } else if (e < 8) {
      w0 = __builtin_amdgcn_alignbit(__float_as_uint(r), w0, 4);
    } else {
      w1 = __builtin_amdgcn_alignbit(__float_as_uint(r), w1, 4);
    }
  }
  if (BITS == 3) w1 >>= 16;
  return make_uint2(w0, w1);
}

template <int KL, int VL>  // levels of the key and value codes
__global__ __launch_bounds__(256) void prefill_kernel(Layout L, const __half *__restrict__ ksrc,
                                                      const __half *__restrict__ vsrc, long long T,
                                                      long long nq) {
  __shared__ __align__(16) __half rows[4][2][8][kRowStride];  // [wave][K|V][token][channel]
  __shared__ unsigned vq[VL == 16 ? 1 : 4][8][8];             // [wave][token i][n]: 16 codes, j-minor
  __shared__ unsigned vqtop[VL == 8 ? 4 : 1][8][8];           // 3-bit codes: their top bits, j-minor
  __shared__ uint2 vq4[VL == 16 ? 4 : 1][8][8 + 1];           // the same for 4-bit codes
  __shared__ unsigned pieces[4][64];
  __shared__ __align__(16) uint8_t units[4][208];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int hk = blockIdx.y, b = blockIdx.z;
  const long long head = (long long)b * L.Hk + hk;
  const long long blk = blockIdx.x;
  const long long t0 = blk * kVBlock + 8 * wave;

  // Source rows (packed row r is token r + S); rows past the end of the prompt are replaced by
  // its last row and never stored.
  {
    const int lr = lane >> 4, lp = lane & 15;
    long long ta = t0 + L.S + lr, tb = t0 + L.S + 4 + lr;
    ta = ta < T ? ta : T - 1;
    tb = tb < T ? tb : T - 1;
    const uint4 *ks = reinterpret_cast<const uint4 *>(ksrc + head * T * kD);
    const uint4 *vs = reinterpret_cast<const uint4 *>(vsrc + head * T * kD);
    const uint4 ka = ks[ta * 16 + lp], kb = ks[tb * 16 + lp];
    const uint4 va = vs[ta * 16 + lp], vb = vs[tb * 16 + lp];
    *reinterpret_cast<uint4 *>(&rows[wave][0][lr][8 * lp]) = ka;
    *reinterpret_cast<uint4 *>(&rows[wave][0][4 + lr][8 * lp]) = kb;
    *reinterpret_cast<uint4 *>(&rows[wave][1][lr][8 * lp]) = va;
    *reinterpret_cast<uint4 *>(&rows[wave][1][4 + lr][8 * lp]) = vb;
  }
  const int i = lane >> 3, n = lane & 7;
  const bool uneq = L.uneq != 0;
  const unsigned gmap = uneq ? L.gmaps[hk] : 0u;
  const int grp = uneq ? tile_group(gmap, n) : (16 * n) / L.G;
  const bool writes_meta = uneq ? (n == 0 || tile_group(gmap, n - 1) != grp) : (16 * n) % L.G == 0;
  const float ak = L.clip_k[hk * L.NG + grp], av = L.clip_v[hk * L.NG + grp];
  int4 pk[4], pv[4];
  {
    const int4 *ppk = reinterpret_cast<const int4 *>(L.perm_k + hk * kD + 16 * n);
    const int4 *ppv = reinterpret_cast<const int4 *>(L.perm_v + hk * kD + 16 * n);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      pk[q] = ppk[q];
      pv[q] = ppv[q];
    }
  }
  const long long t = t0 + i;
  const bool valid = t < nq;
  __syncthreads();

  GroupParams gk, gv;
  constexpr int kKBits = KL == 16 ? 4 : KL == 8 ? 3 : 2, kVBits = VL == 16 ? 4 : VL == 8 ? 3 : 2;
  const uint2 kw = encode16<kKBits>(rows[wave][0][i], pk, ak, L.G, (float)(KL - 1), L.meta_fmt, uneq, gmap, lane, gk);
  const uint2 vw = encode16<kVBits>(rows[wave][1][i], pv, av, L.G, (float)(VL - 1), L.meta_fmt, uneq, gmap, lane, gv);
  unsigned ktop = 0;
  if (KL == 8) {  // the plane dword of a pair of key dwords comes from two lanes
    ktop = place_key_top_bits(kw.y, n & 1);
    ktop |= __shfl_xor(ktop, 1);
  }
  if (valid) {
    if (KL == 16) {
      reinterpret_cast<uint2 *>(L.k_codes + (head * L.Tcap + t) * (kD / 2))[n] = kw;
    } else if (KL == 8) {
      unsigned *krow = reinterpret_cast<unsigned *>(L.k_codes + (head * L.Tcap + t) * 48);
      krow[n] = kw.x;
      if ((n & 1) == 0) krow[8 + (n >> 1)] = ktop;
    } else
      reinterpret_cast<unsigned *>(L.k_codes + (head * L.Tcap + t) * (kD / 4))[n] = kw.x;
    if (writes_meta) {
      meta_store_pair(L.k_meta, (head * L.Tcap + t) * L.NG + grp, MetaPair{gk.scale, gk.lo, gk.stored}, L.meta_fmt);
      meta_store_pair(L.v_meta, (head * L.Tcap + t) * L.NG + grp, MetaPair{gv.scale, gv.lo, gv.stored}, L.meta_fmt);
    }
  }
  // rows past the packed region leave zeros in the block
  if (VL == 16) {
    vq4[wave][i][n] = valid ? vw : make_uint2(0u, 0u);
  } else {
    vq[wave][i][n] = valid ? vw.x : 0u;
    if (VL == 8) vqtop[wave][i][n] = valid ? vw.y : 0u;
  }
  __syncthreads();

  // V units of sub-block kb = wave.  Lane (j = lane % 16, nh = lane / 16) builds fields 2nh and
  // 2nh+1 of unit j from the codes of its eight tokens.
  const int j = lane & 15, nh = lane >> 4;
  uint8_t *dst = L.v_codes + (head * L.n_vblocks + blk) * v_block_bytes_of(VL);
  if (VL == 16) {
    // fields 2nh and 2nh+1 are dwords 2nh and 2nh+1 of the 32-byte unit
    unsigned wa = 0, wb = 0;
#pragma unroll
    for (int ii = 0; ii < 8; ++ii) {
      const uint2 qa = vq4[wave][ii][2 * nh], qb = vq4[wave][ii][2 * nh + 1];
      const unsigned ca = ((j < 8 ? qa.x : qa.y) >> (4 * (j & 7))) & 15u;
      const unsigned cb = ((j < 8 ? qb.x : qb.y) >> (4 * (j & 7))) & 15u;
      wa |= ca << (16 * (ii & 1) + 4 * (ii >> 1));
      wb |= cb << (16 * (ii & 1) + 4 * (ii >> 1));
    }
    reinterpret_cast<uint2 *>(dst + 512 * wave + 32 * j)[nh] = make_uint2(wa, wb);
  } else if (VL == 4 || VL == 8) {
    unsigned w = 0;
#pragma unroll
    for (int ii = 0; ii < 8; ++ii) {
      const unsigned ca = (vq[wave][ii][2 * nh] >> (2 * j)) & 3u;
      const unsigned cb = (vq[wave][ii][2 * nh + 1] >> (2 * j)) & 3u;
      w |= (ca << (16 * (ii & 1) + 2 * (ii >> 1))) | (cb << (8 + 16 * (ii & 1) + 2 * (ii >> 1)));
    }
    if (VL == 4) {
      reinterpret_cast<unsigned *>(dst + 256 * wave)[4 * j + nh] = w;
    } else {
      // 24-byte units: the 2-bit plane, then the two dwords of top bits (fields 4J .. 4J+3 in
      // dword J = nh / 2, built by the lanes nh = 2J and 2J + 1)
      unsigned *unit = reinterpret_cast<unsigned *>(dst + 384 * wave + 24 * j);
      unit[nh] = w;
      unsigned h = 0;
      const int na = (2 * nh) & 3;  // n % 4 of field 2nh; field 2nh+1 has na + 1
#pragma unroll
      for (int ii = 0; ii < 8; ++ii) {
        const unsigned ta = (vqtop[wave][ii][2 * nh] >> j) & 1u;
        const unsigned tb = (vqtop[wave][ii][2 * nh + 1] >> j) & 1u;
        h |= (ta << (16 * (ii & 1) + vtau(na, ii >> 1))) | (tb << (16 * (ii & 1) + vtau(na + 1, ii >> 1)));
      }
      h |= __shfl_xor(h, 16);
      if ((nh & 1) == 0) unit[4 + (nh >> 1)] = h;
    }
  } else {
    unsigned fa = 0, fb = 0, pw = 1;
#pragma unroll
    for (int ii = 0; ii < 8; ++ii) {
      fa += ((vq[wave][ii][2 * nh] >> (2 * j)) & 3u) * pw;
      fb += ((vq[wave][ii][2 * nh + 1] >> (2 * j)) & 3u) * pw;
      pw *= 3;
    }
    pieces[wave][lane] = fa | (fb << 13);  // 26 bits
    __syncthreads();
    if (lane < 16) {
      const unsigned long long a0 = pieces[wave][lane], a1 = pieces[wave][16 + lane];
      const unsigned long long a2 = pieces[wave][32 + lane], a3 = pieces[wave][48 + lane];
      const unsigned long long lo = a0 | (a1 << 26) | (a2 << 52);       // bits 0..63
      const unsigned long long hi = (a2 >> 12) | (a3 << 14);            // bits 64..103
      uint8_t *u = units[wave] + 13 * lane;
#pragma unroll
      for (int q = 0; q < 8; ++q) u[q] = (uint8_t)(lo >> (8 * q));
#pragma unroll
      for (int q = 0; q < 5; ++q) u[8 + q] = (uint8_t)(hi >> (8 * q));
    }
    __syncthreads();
    if (lane < 52)
      reinterpret_cast<unsigned *>(dst + 208 * wave)[lane] = reinterpret_cast<const unsigned *>(units[wave])[lane];
  }
}

// Copies the tokens of the prompt that stay fp16: the last n_win into the ring (token a -> row
// a % W) and the first n_sink into the sink rows (token a -> row W + a).
__global__ __launch_bounds__(64) void ring_fill_kernel(Layout L, const __half *__restrict__ ksrc,
                                                      const __half *__restrict__ vsrc, long long T,
                                                      long long first_win, int n_win) {
  const bool sink = (int)blockIdx.x >= n_win;
  const long long a = sink ? (long long)blockIdx.x - n_win : first_win + blockIdx.x;
  const long long row = sink ? L.W + a : a % L.W;
  const long long head = (long long)blockIdx.z * L.Hk + blockIdx.y;
  const long long src = (head * T + a) * kD, dst = (head * (L.W + L.S) + row) * kD;
  const int lane = threadIdx.x;
  reinterpret_cast<__half2 *>(L.k_win + dst)[lane] = reinterpret_cast<const __half2 *>(ksrc + src)[lane];
  reinterpret_cast<__half2 *>(L.v_win + dst)[lane] = reinterpret_cast<const __half2 *>(vsrc + src)[lane];
}

// ---------------------------------------------------------------------------------------
// Append: one workgroup of two wavefronts per (b, hk); wavefront 0 does K, wavefront 1 does V.
// If the ring is full the slot's old token (number T - W) leaves the window first: a sink token
// is copied to its sink row, any other is quantized into packed row te = T - W - S.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(128) void append_kernel(Layout L, const __half *__restrict__ knew,
                                                     const __half *__restrict__ vnew, long long T) {
  __shared__ __half rows[2][kD];
  __shared__ uint8_t vcodes[kD];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int hk = blockIdx.x, b = blockIdx.y;
  const long long head = (long long)b * L.Hk + hk;
  const long long slot = (head * (L.W + L.S) + T % L.W) * kD;
  const bool leaves = T >= L.W, evict = T - L.W >= L.S;  // a token leaves the window; it is packed
  const long long te = T - L.W - L.S;
  __half *ring = wave ? L.v_win : L.k_win;
  const __half *fresh = (wave ? vnew : knew) + head * kD;

  // Everything the kernel reads is requested up front (one memory round trip): the new token,
  // the slot's old token, the permutation, the clip factor, and what is already stored of the
  // V units the old token will be merged into.
  const __half2 fresh2 = reinterpret_cast<const __half2 *>(fresh)[lane];
  const int s = evict ? (int)(te % kVBlock) : 0, kb = s >> 3, i = s & 7;
  uint8_t *blk = L.v_codes + (head * L.n_vblocks + (evict ? te / kVBlock : 0)) * L.v_block_bytes;
  const bool uneq = L.uneq != 0;
  const unsigned gmap = uneq ? L.gmaps[hk] : 0u;
  const int grp = uneq ? tile_group(gmap, lane >> 3) : (2 * lane) / L.G;
  __half2 old2 = fresh2;
  int p0 = 0, p1 = 0;
  float alpha = 1.f;
  unsigned old_word = 0;   // 2-bit V: dword nh of unit j (lane = (j, nh))
  uint2 old_pair = make_uint2(0u, 0u);  // 4-bit V: dwords 2nh, 2nh+1 of unit j
  unsigned old_top = 0;                 // 3-bit V: dword 4 + nh of unit j (nh < 2)
  uint8_t old_unit[13];    // 3-level V: unit j (lane = j < 16)
#pragma unroll
  for (int q = 0; q < 13; ++q) old_unit[q] = 0;
  if (leaves) old2 = reinterpret_cast<const __half2 *>(ring + slot)[lane];
  if (evict) {
    const int2 pp = reinterpret_cast<const int2 *>((wave ? L.perm_v : L.perm_k) + hk * kD)[lane];
    p0 = pp.x, p1 = pp.y;
    alpha = (wave ? L.clip_v : L.clip_k)[hk * L.NG + grp];
    if (wave == 1 && i != 0) {
      if (L.v_levels == 16) {
        old_pair = reinterpret_cast<const uint2 *>(blk + 32 * (16 * kb + (lane & 15)))[lane >> 4];
      } else if (L.v_levels == 4) {
        old_word = reinterpret_cast<const unsigned *>(blk + 16 * (16 * kb + (lane & 15)))[lane >> 4];
      } else if (L.v_levels == 8) {
        const unsigned *unit = reinterpret_cast<const unsigned *>(blk + 24 * (16 * kb + (lane & 15)));
        old_word = unit[lane >> 4];
        if (lane < 32) old_top = unit[4 + (lane >> 4)];
      } else if (lane < 16) {
        const uint8_t *u = blk + 13 * (16 * kb + lane);
#pragma unroll
        for (int q = 0; q < 13; ++q) old_unit[q] = u[q];
      }
    }
  }
  // the old token is in registers; the new one may take its slot
  reinterpret_cast<__half2 *>(ring + slot)[lane] = fresh2;
  if (leaves && !evict)  // an attention sink: kept as it is
    reinterpret_cast<__half2 *>(ring + (head * (L.W + L.S) + L.W + (T - L.W)) * kD)[lane] = old2;
  if (!evict) return;
  reinterpret_cast<__half2 *>(rows[wave])[lane] = old2;
  __syncthreads();

  const float top = (float)((wave ? L.v_levels : L.k_levels) - 1);
  unsigned c0, c1;
  MetaPair mp;
  encode_row(rows[wave], p0, p1, alpha, L.G, top, L.meta_fmt, uneq, gmap, lane, c0, c1, mp);
  void *meta = wave ? L.v_meta : L.k_meta;
  const bool first_of_group =
      uneq ? ((lane & 7) == 0 && (lane == 0 || tile_group(gmap, (lane >> 3) - 1) != grp)) : (2 * lane) % L.G == 0;
  if (first_of_group)
    meta_store_pair(meta, (head * L.Tcap + te) * L.NG + grp, mp, L.meta_fmt);

  if (wave == 0) {
    uint8_t *krow = L.k_codes + (head * L.Tcap + te) * L.k_row_bytes;
    if (L.k_levels == 16)
      store_k_row4(krow, lane, c0, c1);
    else if (L.k_levels == 8)
      store_k_row3(krow, lane, c0, c1);
    else
      store_k_row(krow, lane, c0, c1);
  } else {
    vcodes[2 * lane] = (uint8_t)c0;
    vcodes[2 * lane + 1] = (uint8_t)c1;
  }
  __syncthreads();
  if (wave == 0) return;

  if (s == 0) {
    // First token of a block: the block starts as zeros.  The 16 units of sub-block 0 are
    // written whole below (i == 0), so only the other three sub-blocks are cleared here.
    const int first = L.v_block_bytes / 16;  // dwords of one sub-block
    for (int w = first + lane; w < L.v_block_bytes / 4; w += 64) reinterpret_cast<unsigned *>(blk)[w] = 0u;
  }
  if (L.v_levels == 16) {
    // lane (j, nh): dwords 2nh and 2nh+1 of unit j are fields 2nh and 2nh+1
    const int j = lane & 15, nh = lane >> 4;
    const unsigned bit = 16 * (i & 1) + 4 * (i >> 1);
    old_pair.x |= (unsigned)vcodes[16 * (2 * nh) + j] << bit;  // old_pair is 0 when i == 0
    old_pair.y |= (unsigned)vcodes[16 * (2 * nh + 1) + j] << bit;
    reinterpret_cast<uint2 *>(blk + 32 * (16 * kb + j))[nh] = old_pair;
  } else if (L.v_levels == 8) {
    // lane (j, nh): dword nh of unit j holds the low two bits of fields 2nh and 2nh+1; the lanes
    // nh < 2 also own dword 4 + nh: the top bits of fields 4nh .. 4nh+3
    const int j = lane & 15, nh = lane >> 4;
    unsigned *unit = reinterpret_cast<unsigned *>(blk + 24 * (16 * kb + j));
    const unsigned bit = 16 * (i & 1) + 2 * (i >> 1);
    const unsigned add = (((unsigned)vcodes[16 * (2 * nh) + j] & 3u) << bit) |
                         (((unsigned)vcodes[16 * (2 * nh + 1) + j] & 3u) << (bit + 8));
    unit[nh] = old_word | add;  // old_word and old_top are 0 when i == 0
    if (nh < 2) {
#pragma unroll
      for (int nn = 0; nn < 4; ++nn)
        old_top |= ((unsigned)vcodes[16 * (4 * nh + nn) + j] >> 2) << (16 * (i & 1) + vtau(nn, i >> 1));
      unit[4 + nh] = old_top;
    }
  } else if (L.v_levels == 4) {
    // lane (j, nh): dword nh of unit j holds fields 2nh and 2nh+1
    const int j = lane & 15, nh = lane >> 4;
    const unsigned bit = 16 * (i & 1) + 2 * (i >> 1);
    const unsigned add = ((unsigned)vcodes[16 * (2 * nh) + j] << bit) | ((unsigned)vcodes[16 * (2 * nh + 1) + j] << (bit + 8));
    reinterpret_cast<unsigned *>(blk + 16 * (16 * kb + j))[nh] = old_word | add;  // old_word is 0 when i == 0
  } else if (lane < 16) {
    const int j = lane;
    uint8_t *u = blk + 13 * (16 * kb + j);
    unsigned long long lo = 0, hi = 0;  // all zero when i == 0
#pragma unroll
    for (int q = 0; q < 8; ++q) lo |= (unsigned long long)old_unit[q] << (8 * q);
#pragma unroll
    for (int q = 0; q < 5; ++q) hi |= (unsigned long long)old_unit[8 + q] << (8 * q);
    unsigned pw = 1;
    for (int q = 0; q < i; ++q) pw *= 3;
    unsigned long long f[8];
    f[0] = lo & 0x1fff; f[1] = (lo >> 13) & 0x1fff; f[2] = (lo >> 26) & 0x1fff; f[3] = (lo >> 39) & 0x1fff;
    f[4] = ((lo >> 52) | (hi << 12)) & 0x1fff; f[5] = (hi >> 1) & 0x1fff; f[6] = (hi >> 14) & 0x1fff;
    f[7] = (hi >> 27) & 0x1fff;
#pragma unroll
    for (int n = 0; n < 8; ++n) f[n] += (unsigned long long)vcodes[16 * n + j] * pw;
    lo = f[0] | (f[1] << 13) | (f[2] << 26) | (f[3] << 39) | (f[4] << 52);
    hi = (f[4] >> 12) | (f[5] << 1) | (f[6] << 14) | (f[7] << 27);
#pragma unroll
    for (int q = 0; q < 8; ++q) u[q] = (uint8_t)(lo >> (8 * q));
#pragma unroll
    for (int q = 0; q < 5; ++q) u[8 + q] = (uint8_t)(hi >> (8 * q));
  }
}

}  // namespace

hipError_t launch_prefill(const Layout &L, const __half *k, const __half *v, long long T, hipStream_t s) {
  const Counts n = counts_of(T, L.W, L.S);
  if (n.n_quant > 0) {
    const long long nblk = (n.n_quant + kVBlock - 1) / kVBlock;
    if (nblk > 0x7fffffffll || L.Hk > 65535 || L.B > 65535) return hipErrorInvalidValue;
    const dim3 grid((unsigned)nblk, L.Hk, L.B), block(256);
#define SKVQ_PREFILL(KL, VL) hipLaunchKernelGGL((prefill_kernel<KL, VL>), grid, block, 0, s, L, k, v, T, n.n_quant)
    if (L.k_levels == 8) {
      if (L.v_levels != 8) return hipErrorInvalidValue;
      SKVQ_PREFILL(8, 8);
    } else if (L.k_levels == 16) {
      if (L.v_levels == 16) SKVQ_PREFILL(16, 16);
      else if (L.v_levels == 4) SKVQ_PREFILL(16, 4);
      else SKVQ_PREFILL(16, 3);
    } else {
      if (L.v_levels == 16) SKVQ_PREFILL(4, 16);
      else if (L.v_levels == 4) SKVQ_PREFILL(4, 4);
      else SKVQ_PREFILL(4, 3);
    }
#undef SKVQ_PREFILL
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const long long n_fp = n.n_win + n.n_sink;
  if (n_fp > 0) {
    if (L.Hk > 65535 || L.B > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(ring_fill_kernel, dim3((unsigned)n_fp, L.Hk, L.B), dim3(64), 0, s, L, k, v, T, T - n.n_win,
                       (int)n.n_win);
    return hipGetLastError();
  }
  return hipSuccess;
}

hipError_t launch_append(const Layout &L, const __half *k_new, const __half *v_new, long long T, hipStream_t s) {
  if (L.B > 65535) return hipErrorInvalidValue;
  hipLaunchKernelGGL(append_kernel, dim3(L.Hk, L.B), dim3(128), 0, s, L, k_new, v_new, T);
  return hipGetLastError();
}

}  // namespace skvq
