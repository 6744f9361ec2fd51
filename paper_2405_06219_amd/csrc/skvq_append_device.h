// Device code of skvq_quantize_append (Section 3.2, decoding phase: the token that slides out of
// the window is quantized, Eq. 2 with the clipped dynamic range of Section 3.1) for gfx950, shared
// by the append kernel and by the decode kernel that takes the new token along.
//
// One wavefront owns one (token, kv head) row; lane l holds the two reordered positions 2l and
// 2l+1 and the group minimum/maximum is a cross-lane butterfly over the lanes of a group.  Every
// fp32 operation of Eq. 2 rounds once: the functions that hold them switch the contraction of
// multiply-add pairs off for themselves, whatever the flags of the file that includes this one.
#pragma once

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
  // (plain operators under the pragma: an operation inside a library intrinsic's body would keep
  // the including file's contraction mode)
#pragma clang fp contract(off)
  if (mn == 0.0f) mn = 0.0f;  // a minimum of -0 is stored as +0
  if (mx == 0.0f) mx = 0.0f;
  GroupParams g;
  const float lo = alpha * mn;
  const float hi = alpha * mx;
  const float range = hi - lo;
  // the codes are computed with the values that decoding will read back from storage
  const MetaPair m = meta_make(range / top, lo, fmt);
  g.lo = m.zero;
  g.scale = m.scale;
  g.stored = m.stored;
  g.inv = g.scale > 0.0f ? 1.0f / g.scale : 0.0f;
  return g;
}

__device__ __forceinline__ unsigned encode(float x, const GroupParams &g, float top) {
#pragma clang fp contract(off)
  const float d = x - g.lo;
  float r = rintf(d * g.inv);
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

// Appends one token per (b, hk): wavefront 0 of the calling workgroup does K, wavefront 1 does V
// (`wave` is the caller's wavefront index; every wavefront of the workgroup must call, the others
// only keep the barriers).  T is the number of tokens cached before the call.  If the ring is full
// the slot's old token (number T - W) leaves the window first: with keep_row >= 0 (a filter rule
// keeps it in full precision) it is copied to row W + keep_row of the fp16 buffers, else it is
// quantized into packed row te.  rows: 2 x 128 halves and vcodes: 128 bytes of LDS.
__device__ __forceinline__ void append_token(const Layout &L, const __half *__restrict__ knew,
                                             const __half *__restrict__ vnew, long long T, int keep_row,
                                             long long te, int hk, int b, int wave, int lane, __half (*rows)[kD],
                                             uint8_t *vcodes) {
  const long long head = (long long)b * L.Hk + hk;
  const long long slot = (head * (L.W + L.S) + T % L.W) * kD;
  const bool leaves = T >= L.W, evict = leaves && keep_row < 0;  // a token leaves the window; it is packed
  if (wave >= 2) {  // (a larger workgroup: the other wavefronts only keep the two barriers below)
    if (evict) {
      __syncthreads();
      __syncthreads();
    }
    return;
  }
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
  if (leaves && !evict)  // kept as it is
    reinterpret_cast<__half2 *>(ring + (head * (L.W + L.S) + L.W + keep_row) * kD)[lane] = old2;
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
}  // namespace skvq
