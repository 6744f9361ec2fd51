// Internal declarations shared by the host API and the HIP kernels of libskvq.
// Not part of the ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "skvq.h"

namespace skvq {

constexpr int kD = 128;        // head dimension
constexpr int kVBlock = 32;    // tokens per V block
constexpr int kTernaryBlockBytes = 832;
constexpr int kTwoBitBlockBytes = 1024;
constexpr int kFourBitBlockBytes = 2048;
constexpr int kThreeBitBlockBytes = 1536;
__host__ __device__ inline int v_block_bytes_of(int levels) {
  return levels == 3 ? kTernaryBlockBytes
         : levels == 16 ? kFourBitBlockBytes
         : levels == 8 ? kThreeBitBlockBytes
                       : kTwoBitBlockBytes;
}
__host__ __device__ inline int k_row_bytes_of(int levels) { return levels == 16 ? 64 : levels == 8 ? 48 : 32; }
constexpr int kPartialStride = kD + 4;  // floats per split partial: m, l, pad, pad, acc[D]

// Everything a kernel needs to find its data; passed by value.
struct Layout {
  int B, Hq, Hk, R;      // R = Hq / Hk
  int G, NG;             // (average) group size, groups per head
  int uneq;              // 1: the groups are unequal (boundaries at multiples of 16 positions)
  const unsigned *gmaps; // device [Hk]: group of the 16 positions 16n .. 16n+15 of a kv head's rows: bits
                         // [4n, 4n+4), n = 0..7 (read only when uneq)
  int W;                 // window
  int S;                 // attention sinks: tokens 0..S-1 are never quantized
  int meta_fmt;          // skvq_meta_format of (scale, zero)
  int k_levels;          // 4, 8 or 16
  int k_row_bytes;       // 32, 48 or 64
  int v_levels;          // 3, 4, 8 or 16
  int v_block_bytes;     // 832, 1024, 1536 or 2048
  long long Tcap;        // packed rows per (b, hk)
  long long n_vblocks;   // ceil(Tcap / 32)
  float sm_scale;
  uint8_t *k_codes, *v_codes;
  void *k_meta, *v_meta;         // (scale, zero) pairs, 8, 4 or 2 bytes each
  __half *k_win, *v_win;         // [B][Hk][W + S][D]: ring rows, then sink rows
  float *workspace;
  const int *perm_k, *perm_v;    // device copies [Hk][D]
  const float *clip_k, *clip_v;  // device copies [Hk][NG]
};

// Where the chunk partials of a decode call are combined.
enum MergeMode {
  kMergeSeparate = 0,  // the chunk kernel writes partials, merge_kernel combines them (a second launch)
  kMergeDirect = 1     // one chunk per kv head: its workgroup writes the output itself
};
struct MergeOut {
  float *out_f32;
  __half *out_f16;  // or null
  int mode;         // MergeMode
};

// Where the T cached tokens of a sequence live (Section 3.2 with the attention-sink rule): the
// last n_win in the ring, of the older ones the first n_sink in sink rows, the other n_quant
// packed (token a is packed row a - S).
struct Counts {
  long long n_win, n_sink, n_quant;
};
// ... with n_kept tokens kept in full precision by the filter rules (whichever they are)
inline Counts counts_with(long long T, int W, long long n_kept) {
  Counts c;
  c.n_win = T < W ? T : W;
  c.n_sink = n_kept;
  c.n_quant = T - c.n_win - n_kept;
  return c;
}
// ... under the attention-sink rule (the first S tokens are kept)
inline Counts counts_of(long long T, int W, int S) {
  Counts c;
  c.n_win = T < W ? T : W;
  const long long old = T - c.n_win;
  c.n_sink = old < S ? old : S;
  c.n_quant = old - c.n_sink;
  return c;
}

// quantize kernels (skvq_quantize.hip)
// n_kept: tokens older than the window that the filter rules keep in fp16 (rows W .. of the fp16
// buffers); kept_ids: device list of their token numbers, ascending, or null for the sink rule
// (tokens 0 .. n_kept-1).
hipError_t launch_prefill(const Layout &L, const __half *k, const __half *v, long long T, long long n_kept,
                          const int *kept_ids, hipStream_t s);
// T: tokens cached before.  The token that leaves the window (if T >= W) goes to fp16 row
// W + keep_row if keep_row >= 0, else to packed row te.
hipError_t launch_append(const Layout &L, const __half *k_new, const __half *v_new, long long T, int keep_row,
                         long long te, hipStream_t s);

// prefill attention (skvq_prefill_attn.hip): causal attention of the prompt on fp16 q, k, v
hipError_t launch_prefill_attention(const Layout &L, const __half *q, const __half *k, const __half *v,
                                    float *out_f32, __half *out_f16, long long T, hipStream_t s);

// clip calibration (skvq_calibrate.hip): err[b * Hk + hk] = squared error of one decode call's
// outputs [B][Hq][D] against ref, over the kv head's query heads and channels
hipError_t launch_sqerr(const Layout &L, const float *out, const float *ref, float *err, hipStream_t s);

// channel reorder (skvq_calibrate.hip): per-chunk (min, max) of every channel, part[((b*Hk + hk)
// * chunks + chunk)][D][2]; KMeans over the reduced statistics (host)
hipError_t launch_channel_stats(const __half *x, float *part, int B, int Hk, long long T, int chunks,
                                hipStream_t s);
int reorder_channels(const float *stats, int Hk, int G, int gran, int max_iter, int32_t *perm, int32_t *bounds);

// decode kernels (skvq_decode.hip)
// n_splits: chunks of the packed region per kv head (>= 1 when n_quant > 0).
// n_new: query tokens per sequence (q, out: [B][n_new][Hq][D]); the last n_new cached tokens are theirs.
// n_kept: tokens kept in fp16 by the filter rules, of the T cached ones.
// k_new, v_new (both or neither): the newest of the T tokens is not in the cache yet, the chunk
// kernel appends it on the way (see append_fusable); the token that leaves the window, if any, is
// packed (n_kept is the same before and after).
hipError_t launch_decode(const Layout &L, const __half *q, float *out_f32, __half *out_f16,
                         long long T, long long n_kept, int n_splits, int n_new, hipStream_t s,
                         const __half *k_new = nullptr, const __half *v_new = nullptr);

// Matrix-core chunk kernel (skvq_decode_mfma.hip): packed chunks and the fp16 tokens (n_sink sink
// rows, then the window's T - nq - n_sink ring tokens); writes partials 0..n_splits-1 (n_splits
// >= 1 even when nothing is packed yet).  A workgroup serves 1, 2 or 4 query heads of a kv head;
// kv heads with 5..8 query heads are read by two workgroups per chunk.
// (n_rows = query heads per kv head x query tokens)
inline int decode_passes(int n_rows) { return n_rows > 4 ? (n_rows + 3) / 4 : 1; }
// te: with knew / vnew, the packed row of the token that leaves the window.
hipError_t launch_decode_mfma(const Layout &L, const __half *q, long long T, long long nq, int n_sink,
                              int n_splits, int n_new, const __half *knew, const __half *vnew, long long te,
                              MergeOut mo, hipStream_t s);
// Whether the decode of T_after tokens (one query token) may append the newest token itself: one
// workgroup per chunk (at most four query heads per kv head), and the token that leaves the
// window, if any, is packed rather than copied to a sink row (a sink row has other readers in
// the same launch).
constexpr int kMinSplitsForOneLaunch = 4;  // chunks per kv head from which the one-launch step is used
inline bool append_fusable(const Layout &L, long long T_after, bool leaving_token_is_kept) {
  const long long T = T_after - 1;  // tokens cached before
  return decode_passes(L.R) == 1 && !(T >= L.W && leaving_token_is_kept);
}
constexpr int kMfmaWavesPerGroup = 8;  // wavefronts per workgroup of the matrix-core kernel

}  // namespace skvq
