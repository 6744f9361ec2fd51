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
#include "skvq_append_device.h"

namespace skvq {
namespace {


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

// The value of another lane of the same row of 16, chosen by a DPP control word.
template <int CTRL>
__device__ __forceinline__ float lane_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// Minimum / maximum of finite numbers as single instructions (fminf / fmaxf first re-canonicalize every
// operand, one more instruction each, for the sake of signalling NaNs that cannot occur here).
__device__ __forceinline__ float min3_raw(float a, float b, float c) {
  float r;
  asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
__device__ __forceinline__ float max3_raw(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
__device__ __forceinline__ float min_raw(float a, float b) {
  float r;
  asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float max_raw(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

// Gathers positions 16n..16n+15 of one parked row into x and finds the group's Eq. 2 parameters.
__device__ __forceinline__ void gather16(const __half *row, const int4 (&pm)[4], float alpha, int G, float top,
                                         int fmt, bool uneq, unsigned gmap, int lane, float (&x)[16],
                                         GroupParams &gp) {
  const int ch[16] = {pm[0].x, pm[0].y, pm[0].z, pm[0].w, pm[1].x, pm[1].y, pm[1].z, pm[1].w,
                      pm[2].x, pm[2].y, pm[2].z, pm[2].w, pm[3].x, pm[3].y, pm[3].z, pm[3].w};
#pragma unroll
  for (int e = 0; e < 16; ++e) x[e] = __half2float(row[ch[e]]);
  float mn = min3_raw(x[0], x[1], x[2]), mx = max3_raw(x[0], x[1], x[2]);
#pragma unroll
  for (int e = 3; e < 15; e += 2) {
    mn = min3_raw(mn, x[e], x[e + 1]);
    mx = max3_raw(mx, x[e], x[e + 1]);
  }
  mn = min_raw(mn, x[15]);
  mx = max_raw(mx, x[15]);
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
    // the group's other lanes are neighbours within eight: lane ^ 1, lane ^ 2, then the mirror
    // image within the eight (both quads hold their own result by then); data-parallel moves
    const int lanes = G / 16;
    if (lanes > 1) {
      mn = min_raw(mn, lane_move<0xB1>(mn));  // quad_perm [1, 0, 3, 2]
      mx = max_raw(mx, lane_move<0xB1>(mx));
    }
    if (lanes > 2) {
      mn = min_raw(mn, lane_move<0x4E>(mn));  // quad_perm [2, 3, 0, 1]
      mx = max_raw(mx, lane_move<0x4E>(mx));
    }
    if (lanes > 4) {
      mn = min_raw(mn, lane_move<0x141>(mn));  // row_half_mirror
      mx = max_raw(mx, lane_move<0x141>(mx));
    }
  }
  gp = group_params(mn, mx, alpha, top, fmt);
}

// code = rint(clamp(y, 0, top)): clamping first gives the same integer because the bounds are
// integers; adding 1.5 * 2^23 rounds to the nearest integer, ties to even, and leaves the code
// in the low bits of the sum.
__device__ __forceinline__ unsigned code_in_low_bits(float x, const GroupParams &gp, float top) {
  const float y = __fmul_rn(__fsub_rn(x, gp.lo), gp.inv);
  return __float_as_uint(__fadd_rn(__builtin_amdgcn_fmed3f(y, 0.0f, top), 12582912.0f));
}

// The 16 codes of a lane as row words.  BITS = 2: two bits each in .x (position 16n + e at bits
// [2e, 2e+2)); BITS = 3: the low two bits like that in .x and the top bits in .y (position e at bit e);
// BITS = 4: four bits each in .x (e = 0..7 at bits [4e, 4e+4)) and .y (e = 8..15).  alignbit shifts
// each code into the word from the top.
template <int BITS>
__device__ __forceinline__ uint2 pack16(const float (&x)[16], const GroupParams &gp, float top) {
  unsigned w0 = 0, w1 = 0;
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const unsigned r = code_in_low_bits(x[e], gp, top);
    if (BITS == 2) {
      w0 = __builtin_amdgcn_alignbit(r, w0, 2);
    } else if (BITS == 3) {
      w0 = __builtin_amdgcn_alignbit(r, w0, 2);
      w1 = __builtin_amdgcn_alignbit(r >> 2, w1, 1);
    } else if (e < 8) {
      w0 = __builtin_amdgcn_alignbit(r, w0, 4);
    } else {
      w1 = __builtin_amdgcn_alignbit(r, w1, 4);
    }
  }
  if (BITS == 3) w1 >>= 16;
  return make_uint2(w0, w1);
}

// Orders a wavefront's own LDS writes before its own later LDS reads (other lanes' data).  The
// LDS serves one wavefront's operations in the order they were issued, so no instruction is
// needed: the fences only keep the compiler from moving the accesses across this point.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// KL, VL: levels of the key and value codes.  PLAIN: the common configuration -- one group per head
// (G = 128), fp32 (scale, zero), kept tokens by the sink rule -- with everything that other
// configurations decide at run time fixed at compile time.
// Grid x: the V blocks, then (first_ring_block on) blocks of four fp16 rows to copy: the last
// n_win tokens into the ring (token a -> row a % W) and the kept ones into the rows after the ring
// (the j-th kept token -> row W + j; it is token kept_ids[j], or token j under the sink rule).
template <int KL, int VL, bool PLAIN>
__global__ __launch_bounds__(256) void prefill_kernel(Layout L, const __half *__restrict__ ksrc,
                                                      const __half *__restrict__ vsrc, long long T,
                                                      long long nq, int n_kept,
                                                      const int *__restrict__ kept_ids_arg,
                                                      unsigned first_ring_block, int n_win) {
  if (blockIdx.x >= first_ring_block) {
    const long long x = 4ll * (blockIdx.x - first_ring_block) + (threadIdx.x >> 6);  // fp16 row: window first, then kept
    if (x >= n_win + n_kept) return;
    const bool kept = x >= n_win;
    const long long j = x - n_win;
    const long long a = kept ? (kept_ids_arg ? (long long)kept_ids_arg[j] : j) : T - n_win + x;
    const long long row = kept ? L.W + j : a % L.W;
    const long long head = (long long)blockIdx.z * L.Hk + blockIdx.y;
    const long long src = (head * T + a) * kD, dst = (head * (L.W + L.S) + row) * kD;
    const int l = threadIdx.x & 63;
    reinterpret_cast<__half2 *>(L.k_win + dst)[l] = reinterpret_cast<const __half2 *>(ksrc + src)[l];
    reinterpret_cast<__half2 *>(L.v_win + dst)[l] = reinterpret_cast<const __half2 *>(vsrc + src)[l];
    return;
  }
  const int *__restrict__ kept_ids = PLAIN ? nullptr : kept_ids_arg;
  const int cfg_G = PLAIN ? kD : L.G, cfg_NG = PLAIN ? 1 : L.NG, cfg_fmt = PLAIN ? (int)SKVQ_META_F32 : L.meta_fmt;
  constexpr bool TERNARY = VL == 3;
  // (everything in LDS is private to one wavefront: the four wavefronts never wait for each other)
  __shared__ __align__(16) __half rows[4][2][8][kRowStride];  // [wave][K|V][token][channel]
  __shared__ unsigned vq[VL == 4 || VL == 8 ? 4 : 1][8][8];   // [wave][token i][n]: 16 codes, j-minor
  __shared__ unsigned vqtop[VL == 8 ? 4 : 1][8][8];           // 3-bit codes: their top bits, j-minor
  __shared__ uint2 vq4[VL == 16 ? 4 : 1][8][8 + 1];           // the same for 4-bit codes
  // ternary codes, one byte each: [wave][position j of the 16][piece n][token i] ...
  __shared__ __align__(16) uint8_t vbytes[TERNARY ? 4 : 1][16][8][8];
  // ... and the 13-bit fields made of them, in the order of the block's bytes: field 8j + n
  __shared__ __align__(4) unsigned short vfields[TERNARY ? 4 : 1][128 + 4];

  // (the wavefront's number in a scalar register: everything derived from it stays scalar)
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int hk = blockIdx.y, b = blockIdx.z;
  const long long head = (long long)b * L.Hk + hk;
  const long long blk = blockIdx.x;
  const long long t0 = blk * kVBlock + 8 * wave;  // first packed row of this wavefront

  // Source rows: packed row r is the r-th token that no filter rule keeps.  With the sink rule
  // (kept_ids == null) the first n_kept tokens are the kept ones: token r + n_kept.  With a list
  // of kept tokens (ascending) token r + (number of j with kept_ids[j] - j <= r); that difference
  // does not decrease with j: binary search.  Rows past the end of the prompt are replaced by
  // its last row and never stored.
  {
    // (the prompt's K and V are read once: streaming loads)
    typedef unsigned u4 __attribute__((ext_vector_type(4)));
    auto stream = [](const uint4 *p) {
      const u4 x = __builtin_nontemporal_load(reinterpret_cast<const u4 *>(p));
      return make_uint4(x.x, x.y, x.z, x.w);
    };
    const int lr = lane >> 4, lp = lane & 15;
    uint4 ka, kb, va, vb;
    if (!kept_ids) {
      // the wavefront's eight rows are one run of the source: a scalar base, lane offsets of 32 bits
      // (rows beyond the prompt's last one repeat it; a run that lies beyond it altogether starts there)
      const long long row0 = t0 + n_kept;                                   // token of packed row t0
      const long long first = row0 < T - 1 ? row0 : T - 1;
      const unsigned last = (unsigned)(T - 1 - first < 7 ? T - 1 - first : 7);  // the prompt's last row, counted from `first`
      const uint4 *ks = reinterpret_cast<const uint4 *>(ksrc + (head * T + first) * kD);
      const uint4 *vs = reinterpret_cast<const uint4 *>(vsrc + (head * T + first) * kD);
      const unsigned oa = 16u * min((unsigned)lr, last) + lp, ob = 16u * min(4u + lr, last) + lp;
      ka = stream(&ks[oa]), kb = stream(&ks[ob]);
      va = stream(&vs[oa]), vb = stream(&vs[ob]);
    } else {
      auto token_of = [&](long long r) {
        int lo = 0, hi = n_kept;  // the count lies in [lo, hi]
        while (lo < hi) {
          const int mid = (lo + hi) >> 1;
          if ((long long)kept_ids[mid] - mid <= r) lo = mid + 1; else hi = mid;
        }
        return r + lo;
      };
      long long ta = token_of(t0 + lr), tb = token_of(t0 + 4 + lr);
      ta = ta < T ? ta : T - 1;
      tb = tb < T ? tb : T - 1;
      const uint4 *ks = reinterpret_cast<const uint4 *>(ksrc + head * T * kD);
      const uint4 *vs = reinterpret_cast<const uint4 *>(vsrc + head * T * kD);
      ka = stream(&ks[ta * 16 + lp]), kb = stream(&ks[tb * 16 + lp]);
      va = stream(&vs[ta * 16 + lp]), vb = stream(&vs[tb * 16 + lp]);
    }
    *reinterpret_cast<uint4 *>(&rows[wave][0][lr][8 * lp]) = ka;
    *reinterpret_cast<uint4 *>(&rows[wave][0][4 + lr][8 * lp]) = kb;
    *reinterpret_cast<uint4 *>(&rows[wave][1][lr][8 * lp]) = va;
    *reinterpret_cast<uint4 *>(&rows[wave][1][4 + lr][8 * lp]) = vb;
  }
  const int i = lane >> 3, n = lane & 7;
  const bool uneq = PLAIN ? false : L.uneq != 0;
  const unsigned gmap = uneq ? L.gmaps[hk] : 0u;
  const int grp = uneq ? tile_group(gmap, n) : (16 * n) / cfg_G;
  const bool writes_meta = uneq ? (n == 0 || tile_group(gmap, n - 1) != grp) : (16 * n) % cfg_G == 0;
  const float ak = L.clip_k[hk * cfg_NG + grp], av = L.clip_v[hk * cfg_NG + grp];
  int4 pk[4], pv[4];
  {
    const int4 *ppk = reinterpret_cast<const int4 *>(L.perm_k + hk * kD) + 4 * n;
    const int4 *ppv = reinterpret_cast<const int4 *>(L.perm_v + hk * kD) + 4 * n;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      pk[q] = ppk[q];
      pv[q] = ppv[q];
    }
  }
  // the wavefront's rows that exist: rows t0 .. t0 + n_valid - 1 (rows past the packed region are
  // computed from the stand-in data and dropped)
  const int n_valid = (int)(nq - t0 < 8 ? (nq - t0 < 0 ? 0 : nq - t0) : 8);
  const bool valid = i < n_valid;
  wave_lds_sync();

  GroupParams gk, gv;
  constexpr int kKBits = KL == 16 ? 4 : KL == 8 ? 3 : 2, kVBits = VL == 16 ? 4 : VL == 8 ? 3 : 2;
  float x[16];
  gather16(rows[wave][0][i], pk, ak, cfg_G, (float)(KL - 1), cfg_fmt, uneq, gmap, lane, x, gk);
  const uint2 kw = pack16<kKBits>(x, gk, (float)(KL - 1));
  gather16(rows[wave][1][i], pv, av, cfg_G, (float)(VL - 1), cfg_fmt, uneq, gmap, lane, x, gv);
  uint2 vw = make_uint2(0u, 0u);
  if constexpr (TERNARY) {
    // the sum's low byte is the code: sixteen byte stores, no packing
    uint8_t *col = &vbytes[wave][0][n][i];
#pragma unroll
    for (int e = 0; e < 16; ++e) col[64 * e] = (uint8_t)code_in_low_bits(x[e], gv, 2.0f);
  } else {
    vw = pack16<kVBits>(x, gv, (float)(VL - 1));
  }
  unsigned ktop = 0;
  if (KL == 8) {  // the plane dword of a pair of key dwords comes from two lanes
    ktop = place_key_top_bits(kw.y, n & 1);
    ktop |= __shfl_xor(ktop, 1);
  }
  // packed key rows and (scale, zero) pairs of the wavefront's rows: scalar bases at row t0, the
  // lane's row and piece as 32-bit offsets
  if (valid) {
    uint8_t *krows = L.k_codes + (head * L.Tcap + t0) * k_row_bytes_of(KL);
    if (KL == 16) {
      reinterpret_cast<uint2 *>(krows)[lane] = kw;  // row i, dwords 2n and 2n+1
    } else if (KL == 8) {
      unsigned *krow = reinterpret_cast<unsigned *>(krows) + 12 * i;
      krow[n] = kw.x;
      if ((n & 1) == 0) krow[8 + (n >> 1)] = ktop;
    } else
      __builtin_nontemporal_store(kw.x, reinterpret_cast<unsigned *>(krows) + lane);  // row i, dword n
    if (writes_meta) {
      const size_t pair_bytes = cfg_fmt == SKVQ_META_F32 ? 8 : cfg_fmt == SKVQ_META_F16 ? 4 : 2;
      const size_t first = (size_t)(head * L.Tcap + t0) * cfg_NG * pair_bytes;
      meta_store_pair(reinterpret_cast<uint8_t *>(L.k_meta) + first, i * cfg_NG + grp, MetaPair{gk.scale, gk.lo, gk.stored}, cfg_fmt);
      meta_store_pair(reinterpret_cast<uint8_t *>(L.v_meta) + first, i * cfg_NG + grp, MetaPair{gv.scale, gv.lo, gv.stored}, cfg_fmt);
    }
  }
  // rows past the packed region leave zeros in the block
  if (VL == 16) {
    vq4[wave][i][n] = valid ? vw : make_uint2(0u, 0u);
  } else if (!TERNARY) {
    vq[wave][i][n] = valid ? vw.x : 0u;
    if (VL == 8) vqtop[wave][i][n] = valid ? vw.y : 0u;
  }
  wave_lds_sync();

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
    // A field is the base-3 number whose digit i is token i's code: the codes of tokens 0..3 and 4..7
    // arrive as the bytes of two dwords, and a byte-wise dot product with (1, 3, 9, 27) sums four
    // digits at once.
    uint4 c = *reinterpret_cast<const uint4 *>(&vbytes[wave][j][2 * nh][0]);
    if (n_valid < 8) {  // (a scalar condition) bytes of rows that do not exist count as zero
      const unsigned lo = n_valid >= 4 ? ~0u : (1u << (8 * n_valid)) - 1u;
      const unsigned hi = n_valid <= 4 ? 0u : (1u << (8 * (n_valid - 4))) - 1u;
      c.x &= lo, c.z &= lo, c.y &= hi, c.w &= hi;
    }
    constexpr unsigned kPowers = 1u | (3u << 8) | (9u << 16) | (27u << 24);
    const unsigned fa = __builtin_amdgcn_udot4(c.x, kPowers, __umul24(81u, __builtin_amdgcn_udot4(c.y, kPowers, 0u, false)), false);
    const unsigned fb = __builtin_amdgcn_udot4(c.z, kPowers, __umul24(81u, __builtin_amdgcn_udot4(c.w, kPowers, 0u, false)), false);
    reinterpret_cast<unsigned *>(vfields[wave])[4 * j + nh] = fa | (fb << 16);  // fields 8j + 2nh and the next
    wave_lds_sync();
    // The sub-block's 208 bytes are its 128 fields of 13 bits in a row.  Lane d < 52 builds dword d:
    // bits 32d .. 32d+31 lie in the four fields from number 32d / 13 on.
    if (lane < 52) {
      const unsigned first = (32u * lane) / 13u, shift = 32u * lane - 13u * first;
      const unsigned short *f = &vfields[wave][first];
      const unsigned f0 = f[0], f1 = f[1], f2 = f[2], f3 = f[3];  // (f3 of the last dword is padding, shifted out)
      const unsigned low = f0 | (f1 << 13) | (f2 << 26), high = (f2 >> 6) | (f3 << 7);  // bits 0..31 and 32..51
      __builtin_nontemporal_store(__builtin_amdgcn_alignbit(high, low, shift), reinterpret_cast<unsigned *>(dst + 208 * wave) + lane);
    }
  }
}

// Append: one workgroup of two wavefronts per (b, hk) (skvq_append_device.h).
__global__ __launch_bounds__(128) void append_kernel(Layout L, const __half *__restrict__ knew,
                                                     const __half *__restrict__ vnew, long long T, int keep_row,
                                                     long long te) {
  __shared__ __half rows[2][kD];
  __shared__ uint8_t vcodes[kD];
  append_token(L, knew, vnew, T, keep_row, te, blockIdx.x, blockIdx.y, threadIdx.x >> 6, threadIdx.x & 63, rows,
               vcodes);
}

}  // namespace

hipError_t launch_prefill(const Layout &L, const __half *k, const __half *v, long long T, long long n_kept,
                          const int *kept_ids, hipStream_t s) {
  const Counts n = counts_with(T, L.W, n_kept);
  if (n_kept < 0 || n_kept > L.S || n.n_quant < 0) return hipErrorInvalidValue;
  const long long nblk = (n.n_quant + kVBlock - 1) / kVBlock;       // V blocks of packed rows
  const long long n_fp = n.n_win + n.n_sink, ring_blocks = (n_fp + 3) / 4;  // fp16 rows, four per workgroup
  if (nblk + ring_blocks == 0) return hipSuccess;
  if (nblk + ring_blocks > 0x7fffffffll || L.Hk > 65535 || L.B > 65535) return hipErrorInvalidValue;
  const dim3 grid((unsigned)(nblk + ring_blocks), L.Hk, L.B), block(256);
  const bool plain = L.NG == 1 && !L.uneq && L.meta_fmt == SKVQ_META_F32 && kept_ids == nullptr;
#define SKVQ_PREFILL_P(KL, VL, PP)                                                                             \
  hipLaunchKernelGGL((prefill_kernel<KL, VL, PP>), grid, block, 0, s, L, k, v, T, n.n_quant, (int)n_kept, kept_ids, \
                     (unsigned)nblk, (int)n.n_win)
#define SKVQ_PREFILL(KL, VL) \
  if (plain) SKVQ_PREFILL_P(KL, VL, true); else SKVQ_PREFILL_P(KL, VL, false)
  if (L.k_levels == 8) {
    if (L.v_levels != 8) return hipErrorInvalidValue;
    SKVQ_PREFILL(8, 8);
  } else if (L.k_levels == 16) {
    if (L.v_levels == 16) { SKVQ_PREFILL(16, 16); }
    else if (L.v_levels == 4) { SKVQ_PREFILL(16, 4); }
    else { SKVQ_PREFILL(16, 3); }
  } else {
    if (L.v_levels == 16) { SKVQ_PREFILL(4, 16); }
    else if (L.v_levels == 4) { SKVQ_PREFILL(4, 4); }
    else { SKVQ_PREFILL(4, 3); }
  }
#undef SKVQ_PREFILL
#undef SKVQ_PREFILL_P
  return hipGetLastError();
}

hipError_t launch_append(const Layout &L, const __half *k_new, const __half *v_new, long long T, int keep_row,
                         long long te, hipStream_t s) {
  if (L.B > 65535 || keep_row >= L.S || (T >= L.W && keep_row < 0 && (te < 0 || te >= L.Tcap))) return hipErrorInvalidValue;
  hipLaunchKernelGGL(append_kernel, dim3(L.Hk, L.B), dim3(128), 0, s, L, k_new, v_new, T, keep_row, te);
  return hipGetLastError();
}

}  // namespace skvq
