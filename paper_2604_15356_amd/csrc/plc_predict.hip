// Floating-point half of the codec: top-k prediction, residual, quantiser
// (encode) and dequantise / add-back (decode).  See include/plc.h for the
// definition of every step; the paper passages are Sec. 7.1 ("Top-k
// approximation"), Def. "KV residual" and Sec. 7.2 (the two integration
// points of the inference loop).
//
// Both directions are HBM streams: per KV component they read 2k bytes of
// candidates and touch 3 more bytes, with about 2k + 20 fp32 operations in
// between.  There is no data reuse and no contraction, so the kernels are
// organised purely around wide coalesced accesses: one thread owns one
// 16-byte chunk (8 components) of one K or V row, and issues all of its
// k + 1 loads before the first use.
#include <mutex>

#include "plc_device.h"

namespace plc {
namespace {

// Escapes of a tile are first parked in a per-tile staging row of this many entries (a tile has 2048
// symbols; the synthetic workloads escape 0.7 % of them).  A tile with more escapes than that is
// gathered again from its symbols by the compaction pass.
constexpr int kEscStage = 128;

struct CodecArgs {
  const uint16_t *cand_k, *cand_v;
  const uint16_t *act_k, *act_v;  // encode only
  uint16_t *out_k, *out_v;        // decode only
  const float *weights;           // [S, n, k] renormalised weights
  const int32_t *chosen;          // [S, n] index of the true candidate or -1 (token-conditional calls only)
  const uint8_t *bits;            // [S, n] bit depth of the position (adaptive calls only)
  float range;                    // adaptive calls: step = range * 2^-bits
  uint8_t *symbols;               // encode: out, decode: in
  const uint16_t *esc_in;         // decode
  uint64_t esc_len;               // decode
  const uint64_t *esc_off;        // decode
  float *pred_out;                // encode, nullable
  uint32_t *counts;               // encode, nullable: [n_streams, 256] symbol counts taken on the way
  uint32_t *tile_cnt;             // [n_streams * tiles_per_stream] escapes per tile
  uint16_t *esc_stage;            // encode: [n_tiles, kEscStage] escapes of each tile in symbol order
  const uint32_t *tile_off;       // decode: exclusive prefix of tile_cnt inside a stream
  uint32_t *status;
  int32_t L, H, n, k, d8;
  uint32_t tiles_per_stream, chunks_per_stream;
  int64_t cs[5], as[4];
  int64_t syms_per_stream;
  float delta, qmax;
};

// Where a thread's chunk lives.  All threads of a workgroup share (s, l, h).
struct Coord {
  bool valid;
  int64_t cand;  // element offset of candidate 0, component 0 of the chunk
  int64_t act;   // element offset in act / out
  int64_t w;     // offset of the weight row
  int64_t row;   // s * n + i, the position's entry in per-position arrays
  int64_t sym;   // offset in symbols / pred_out
  int c;         // 0 = K, 1 = V
  uint32_t stream, tile;
};

__device__ __forceinline__ Coord locate_chunk(const CodecArgs &a, uint32_t stream, uint32_t tile, uint32_t slot) {
  Coord q;
  q.stream = stream;
  q.tile = tile;
  const uint32_t lh = a.L * a.H;
  const uint32_t s = q.stream / lh;
  const uint32_t r = q.stream - s * lh;
  const uint32_t l = r / a.H;
  const uint32_t h = r - l * a.H;
  const uint32_t chunk = q.tile * kBlock + slot;  // slot: which of the tile's 256 chunks
  q.valid = chunk < a.chunks_per_stream;
  const uint32_t row = chunk / (uint32_t)a.d8;  // row = i * 2 + c
  const uint32_t e8 = chunk - row * a.d8;
  const uint32_t i = row >> 1;
  q.c = row & 1;
  q.cand = s * a.cs[0] + l * a.cs[1] + h * a.cs[2] + (int64_t)i * a.cs[3] + e8 * kChunk;
  q.act = s * a.as[0] + l * a.as[1] + h * a.as[2] + (int64_t)i * a.as[3] + e8 * kChunk;
  q.row = (int64_t)s * a.n + i;
  q.w = q.row * a.k;
  q.sym = (int64_t)q.stream * a.syms_per_stream + (int64_t)chunk * kChunk;
  return q;
}

// One workgroup per tile, one thread per chunk.
__device__ __forceinline__ Coord locate(const CodecArgs &a) {
  const uint32_t stream = blockIdx.x / a.tiles_per_stream;
  return locate_chunk(a, stream, blockIdx.x - stream * a.tiles_per_stream, threadIdx.x);
}

// pred[e] = sum_j w[j] * cand_j[e], fp32 fused multiply-add, j ascending from 0.
template <int K>
__device__ __forceinline__ void predict8(const uint16_t *cand, int64_t sj, const float *w, int k,
                                         float pred[kChunk]) {
#pragma unroll
  for (int e = 0; e < kChunk; ++e) pred[e] = 0.0f;
  if constexpr (K > 0) {
    uint4 cv[K];
    float wv[K];
#pragma unroll
    for (int j = 0; j < K; ++j) cv[j] = load16_stream(cand + j * sj);
#pragma unroll
    for (int j = 0; j < K; ++j) wv[j] = w[j];
#pragma unroll
    for (int j = 0; j < K; ++j) accumulate8(wv[j], cv[j], pred);
  } else {
#pragma unroll 4
    for (int j = 0; j < k; ++j) accumulate8(w[j], load16_stream(cand + j * sj), pred);
  }
}

// Quantiser step of a chunk's position: the configured one, or range * 2^-b for the adaptive calls.
__device__ __forceinline__ float position_step(const CodecArgs &a, int64_t row) {
  if (!a.bits) return a.delta;
  int b = a.bits[row];
  if (b < 1 || b > PLC_MAX_BITS) {
    raise(a.status, PLC_ERR_INVALID);
    b = 1;
  }
  return __builtin_ldexpf(a.range, -b);
}

// The prediction of one chunk.  COND: the position names its true candidate, whose vector then is the
// prediction (Lemma "KV determinism"); -1 falls back to the weighted mean.
template <int K, bool COND>
__device__ __forceinline__ void predict_chunk(const CodecArgs &a, const Coord &q, const uint16_t *cand,
                                              float pred[kChunk]) {
  if constexpr (COND) {
    int pick = a.chosen[q.row];
    if (pick < -1 || pick >= a.k) {
      raise(a.status, PLC_ERR_INVALID);
      pick = -1;
    }
    if (pick >= 0) {
      const half8 c = __builtin_bit_cast(half8, load16_stream(cand + pick * a.cs[4]));
#pragma unroll
      for (int e = 0; e < kChunk; ++e) pred[e] = (float)c[e];
      return;
    }
  }
  predict8<K>(cand, a.cs[4], a.weights + q.w, a.k, pred);
}

// ---------------------------------------------------------------------------
// w[s,i,j] = p[s,i,j] / sum_m p[s,i,m]   (one thread per probability row)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void weights_kernel(const float *__restrict__ probs, float *__restrict__ w,
                                                         int64_t rows, int k, uint32_t *status) {
  const int64_t row = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (row >= rows) return;
  const float *p = probs + row * k;
  float Z = 0.0f;
  bool bad = false;
  for (int j = 0; j < k; ++j) {
    const float pj = p[j];
    if (!(pj >= 0.0f)) bad = true;  // negative or NaN
    Z = Z + pj;
  }
  if (!(Z > 0.0f) || __builtin_isinf(Z)) bad = true;
  for (int j = 0; j < k; ++j) w[row * k + j] = bad ? 0.0f : p[j] / Z;
  if (bad) raise(status, PLC_ERR_INVALID);
}

// ---------------------------------------------------------------------------
// Encode: symbols and per-tile escape counts
// ---------------------------------------------------------------------------
// Residual of one chunk against its prediction, quantised: the 8 symbols packed low byte first, the number
// of escapes among them and a bit mask of which.
__device__ __forceinline__ void quantise8(const half8 x, const float pred[kChunk], float delta, float qmax,
                                          uint32_t packed[2], uint32_t *n_esc, uint32_t *esc_bits) {
  packed[0] = packed[1] = 0u;
#pragma unroll
  for (int e = 0; e < kChunk; ++e) {
    const float r = (float)x[e] - pred[e];
    const float u = r / delta;
    const float qf = __builtin_rintf(u);  // round half to even
    uint32_t sym;
    if (__builtin_fabsf(qf) <= qmax) {  // false for NaN and infinities
      sym = (uint32_t)((int)qf + (int)kZeroSymbol);
    } else {
      sym = PLC_ESCAPE;
      *n_esc += 1;
      *esc_bits |= 1u << e;
    }
    packed[e >> 2] |= sym << (8 * (e & 3));
  }
}

// Park a thread's escapes (raw fp16 of the actual values) in the tile's staging row from position `pos` on.
__device__ __forceinline__ void stage_escapes(uint16_t *row, uint32_t pos, uint32_t esc_bits, const uint4 av) {
  const uint32_t raw[4] = {av.x, av.y, av.z, av.w};
#pragma unroll
  for (int e = 0; e < kChunk; ++e) {
    if (esc_bits & (1u << e)) {
      if (pos < (uint32_t)kEscStage) row[pos] = (uint16_t)((e & 1 ? raw[e >> 1] >> 16 : raw[e >> 1]) & 0xffffu);
      ++pos;
    }
  }
}

template <int K>
__global__ __launch_bounds__(kBlock) void predict_residual_kernel(const CodecArgs a) {
  __shared__ uint32_t wave_cnt[kBlock / 64];
  const Coord q = locate(a);
  uint32_t n_esc = 0, esc_bits = 0;
  uint4 av = make_uint4(0u, 0u, 0u, 0u);
  if (q.valid) {
    const uint16_t *cand = (q.c ? a.cand_v : a.cand_k) + q.cand;
    const uint16_t *act = (q.c ? a.act_v : a.act_k) + q.act;
    av = load16_stream(act);
    float pred[kChunk];
    predict8<K>(cand, a.cs[4], a.weights + q.w, a.k, pred);
    uint32_t packed[2];
    quantise8(__builtin_bit_cast(half8, av), pred, a.delta, a.qmax, packed, &n_esc, &esc_bits);
    store8_stream(a.symbols + q.sym, packed[0], packed[1]);
    if (a.pred_out) {
      float4 *po = reinterpret_cast<float4 *>(a.pred_out + q.sym);
      po[0] = make_float4(pred[0], pred[1], pred[2], pred[3]);
      po[1] = make_float4(pred[4], pred[5], pred[6], pred[7]);
    }
  }
  // Escapes of this tile, in symbol order, go to the tile's staging row; a later sparse pass moves
  // them to their final place once the counts of all tiles in front are known.
  uint32_t wave_total = 0, prefix = 0;
  if (__ballot(n_esc != 0) != 0) prefix = wave_escape_prefix(n_esc, &wave_total);  // uniform
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) wave_cnt[wave] = wave_total;
  __syncthreads();
  const uint32_t c0 = wave_cnt[0], c1 = wave_cnt[1], c2 = wave_cnt[2], c3 = wave_cnt[3];
  if (threadIdx.x == 0) a.tile_cnt[blockIdx.x] = c0 + c1 + c2 + c3;
  if (n_esc) {
    const uint32_t pos = prefix + (wave > 0 ? c0 : 0u) + (wave > 1 ? c1 : 0u) + (wave > 2 ? c2 : 0u);
    stage_escapes(a.esc_stage + (int64_t)blockIdx.x * kEscStage, pos, esc_bits, av);
  }
}

// The same pass with the symbol statistics taken on the way (plc_predict_residual_hist): a workgroup counts
// every symbol it produces in a histogram in LDS (one copy per wavefront; LDS atomics, a few hundred cycles per
// tile against the ~4000 the tile's bytes take to arrive) and at the end adds its non-empty bins to the
// stream's counts with global atomics -- integer adds, so the result does not depend on the order.  The
// symbols are then not read back for a histogram pass of their own (1 byte per component and a launch).
// One tile per workgroup, as in the kernel above, measured best (64 sessions: the call 28.3 -> 28.4 ms against
// 2.3 ms for the histogram pass it replaces; Llama shape 0.84 -> 0.88 against 0.08): walking several tiles in
// one workgroup saves global atomics but puts a barrier between the tiles' loads (4 tiles: 29.6 and 0.94 ms).
// Only where a stream is so long that thousands of workgroups in flight add to the same 256 counters do two
// tiles per workgroup pay (32,768 positions, 4096 tiles per stream: 4.8 -> 4.4 ms).
constexpr int kHistLongStream = 1024;  // tiles per stream from which on a workgroup takes two

template <int K>
__global__ __launch_bounds__(kBlock) void predict_residual_hist_kernel(const CodecArgs a, uint32_t *__restrict__ counts,
                                                                       uint32_t wgs_per_stream, uint32_t tiles_per_wg) {
  __shared__ uint32_t hist[kBlock / 64][256];
  __shared__ uint32_t wave_cnt[2][kBlock / 64];
  const uint32_t stream = blockIdx.x / wgs_per_stream;
  const uint32_t first_tile = (blockIdx.x - stream * wgs_per_stream) * tiles_per_wg;
  const int wave = threadIdx.x >> 6;
#pragma unroll
  for (int w = 0; w < kBlock / 64; ++w) hist[w][threadIdx.x] = 0u;
  __syncthreads();
  uint32_t *myhist = hist[wave];
#pragma unroll 1
  for (uint32_t t = 0; t < tiles_per_wg; ++t) {
    const uint32_t tile = first_tile + t;
    if (tile >= a.tiles_per_stream) break;  // uniform
    const int64_t g = (int64_t)stream * a.tiles_per_stream + tile;  // the tile's place in the per-tile arrays
    const Coord q = locate_chunk(a, stream, tile, threadIdx.x);
    uint32_t n_esc = 0, esc_bits = 0;
    uint4 av = make_uint4(0u, 0u, 0u, 0u);
    if (q.valid) {
      const uint16_t *cand = (q.c ? a.cand_v : a.cand_k) + q.cand;
      const uint16_t *act = (q.c ? a.act_v : a.act_k) + q.act;
      av = load16_stream(act);
      float pred[kChunk];
      predict8<K>(cand, a.cs[4], a.weights + q.w, a.k, pred);
      uint32_t packed[2];
      quantise8(__builtin_bit_cast(half8, av), pred, a.delta, a.qmax, packed, &n_esc, &esc_bits);
      store8_stream(a.symbols + q.sym, packed[0], packed[1]);
      if (a.pred_out) {
        float4 *po = reinterpret_cast<float4 *>(a.pred_out + q.sym);
        po[0] = make_float4(pred[0], pred[1], pred[2], pred[3]);
        po[1] = make_float4(pred[4], pred[5], pred[6], pred[7]);
      }
#pragma unroll
      for (int e = 0; e < kChunk; ++e) atomicAdd(&myhist[(packed[e >> 2] >> (8 * (e & 3))) & 255u], 1u);
    }
    uint32_t wave_total = 0, prefix = 0;
    if (__ballot(n_esc != 0) != 0) prefix = wave_escape_prefix(n_esc, &wave_total);  // uniform
    uint32_t *cnt = wave_cnt[t & 1];  // two rows in turn: one barrier per tile is enough
    if ((threadIdx.x & 63) == 0) cnt[wave] = wave_total;
    __syncthreads();
    const uint32_t c0 = cnt[0], c1 = cnt[1], c2 = cnt[2], c3 = cnt[3];
    if (threadIdx.x == 0) a.tile_cnt[g] = c0 + c1 + c2 + c3;
    if (n_esc) {
      const uint32_t pos = prefix + (wave > 0 ? c0 : 0u) + (wave > 1 ? c1 : 0u) + (wave > 2 ? c2 : 0u);
      stage_escapes(a.esc_stage + g * kEscStage, pos, esc_bits, av);
    }
  }
  __syncthreads();
  const uint32_t v = hist[0][threadIdx.x] + hist[1][threadIdx.x] + hist[2][threadIdx.x] + hist[3][threadIdx.x];
  if (v) atomicAdd(&counts[(int64_t)stream * 256 + threadIdx.x], v);
  static_assert(kBlock == 256, "one thread per bin");
}

__global__ __launch_bounds__(kBlock) void zero_counts_kernel(uint32_t *__restrict__ p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// Token-conditional encode.  A position whose token is a candidate reads 2 bytes per component of that
// candidate instead of 2k of all of them, so a thread has only two loads to keep in flight per chunk; a
// workgroup therefore takes kCondTiles consecutive tiles and issues the loads of all of them first (two
// tiles measured best; with four the quantiser's arithmetic, 8 IEEE divides per chunk, starts to queue
// behind the loads instead of overlapping them).
constexpr int kCondTiles = 2;

template <int K>
__global__ __launch_bounds__(kBlock) void predict_residual_cond_kernel(const CodecArgs a, uint32_t n_tiles) {
  __shared__ uint32_t wave_cnt[kCondTiles][kBlock / 64];
  Coord q[kCondTiles];
  uint4 av[kCondTiles], cv[kCondTiles];
  int pick[kCondTiles];
#pragma unroll
  for (int t = 0; t < kCondTiles; ++t) {
    const uint32_t g = blockIdx.x * kCondTiles + t;
    const bool inside = g < n_tiles;  // uniform
    const uint32_t gg = inside ? g : 0u;
    const uint32_t stream = gg / a.tiles_per_stream;
    q[t] = locate_chunk(a, stream, gg - stream * a.tiles_per_stream, threadIdx.x);
    q[t].valid = q[t].valid && inside;
    av[t] = cv[t] = make_uint4(0u, 0u, 0u, 0u);
    pick[t] = -1;
    if (q[t].valid) {
      av[t] = load16_stream((q[t].c ? a.act_v : a.act_k) + q[t].act);
      pick[t] = a.chosen[q[t].row];
    }
  }
#pragma unroll
  for (int t = 0; t < kCondTiles; ++t) {
    if (pick[t] < -1 || pick[t] >= a.k) {
      raise(a.status, PLC_ERR_INVALID);
      pick[t] = -1;
    }
    if (pick[t] >= 0) cv[t] = load16_stream((q[t].c ? a.cand_v : a.cand_k) + q[t].cand + pick[t] * a.cs[4]);
  }
  uint32_t n_esc[kCondTiles], esc_bits[kCondTiles], prefix[kCondTiles];
  const int wave = threadIdx.x >> 6;
#pragma unroll
  for (int t = 0; t < kCondTiles; ++t) {
    n_esc[t] = esc_bits[t] = 0;
    if (q[t].valid) {
      float pred[kChunk];
      if (pick[t] >= 0) {
        const half8 c = __builtin_bit_cast(half8, cv[t]);
#pragma unroll
        for (int e = 0; e < kChunk; ++e) pred[e] = (float)c[e];
      } else {
        predict8<K>((q[t].c ? a.cand_v : a.cand_k) + q[t].cand, a.cs[4], a.weights + q[t].w, a.k, pred);
      }
      uint32_t packed[2];
      quantise8(__builtin_bit_cast(half8, av[t]), pred, position_step(a, q[t].row), a.qmax, packed, &n_esc[t],
                &esc_bits[t]);
      store8_stream(a.symbols + q[t].sym, packed[0], packed[1]);
      if (a.pred_out) {
        float4 *po = reinterpret_cast<float4 *>(a.pred_out + q[t].sym);
        po[0] = make_float4(pred[0], pred[1], pred[2], pred[3]);
        po[1] = make_float4(pred[4], pred[5], pred[6], pred[7]);
      }
    }
    uint32_t wave_total = 0;
    prefix[t] = 0;
    if (__ballot(n_esc[t] != 0) != 0) prefix[t] = wave_escape_prefix(n_esc[t], &wave_total);  // uniform
    if ((threadIdx.x & 63) == 0) wave_cnt[t][wave] = wave_total;
  }
  __syncthreads();
#pragma unroll
  for (int t = 0; t < kCondTiles; ++t) {
    const uint32_t g = blockIdx.x * kCondTiles + t;
    if (g >= n_tiles) break;
    const uint32_t c0 = wave_cnt[t][0], c1 = wave_cnt[t][1], c2 = wave_cnt[t][2], c3 = wave_cnt[t][3];
    if (threadIdx.x == 0) a.tile_cnt[g] = c0 + c1 + c2 + c3;
    if (n_esc[t]) {
      const uint32_t pos = prefix[t] + (wave > 0 ? c0 : 0u) + (wave > 1 ? c1 : 0u) + (wave > 2 ? c2 : 0u);
      stage_escapes(a.esc_stage + (int64_t)g * kEscStage, pos, esc_bits[t], av[t]);
    }
  }
}

// Count the escape symbols of each tile (decode side).  One wavefront per tile, 32 bytes per lane: a tile per
// workgroup would spend its time starting workgroups, this way the pass runs at memory speed.
__global__ __launch_bounds__(kBlock) void count_escapes_kernel(const CodecArgs a, uint32_t n_tiles) {
  const uint32_t t = blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);  // tile, uniform per wavefront
  if (t >= n_tiles) return;
  const int lane = threadIdx.x & 63;
  const uint32_t stream = t / a.tiles_per_stream;
  const uint32_t tile = t - stream * a.tiles_per_stream;
  const uint32_t chunk0 = tile * kBlock + lane * 4;  // this lane's four chunks of 8 symbols
  const uint8_t *p = a.symbols + (int64_t)stream * a.syms_per_stream + (int64_t)chunk0 * kChunk;
  uint32_t n_esc = 0;
#pragma unroll
  for (int c = 0; c < 4; ++c) {  // 8-byte loads: that is the alignment the symbols are promised to have
    if (chunk0 + c < a.chunks_per_stream) {
      const uint2 v = *reinterpret_cast<const uint2 *>(p + kChunk * c);
      // a byte is 0xff iff its low seven bits carry into bit 7 when 1 is added and bit 7 is set
      n_esc += (uint32_t)__builtin_popcount(((v.x & 0x7f7f7f7fu) + 0x01010101u) & v.x & 0x80808080u);
      n_esc += (uint32_t)__builtin_popcount(((v.y & 0x7f7f7f7fu) + 0x01010101u) & v.y & 0x80808080u);
    }
  }
  static_assert(PLC_ESCAPE == 255, "the byte test above");
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) n_esc += __shfl_xor(n_esc, off, 64);
  if (lane == 0) a.tile_cnt[t] = n_esc;
}

// Exclusive prefix sum of the tile counts inside each stream; one workgroup per stream.
__global__ __launch_bounds__(kBlock) void scan_tiles_kernel(const uint32_t *__restrict__ tile_cnt,
                                                            uint32_t *__restrict__ tile_off,
                                                            uint32_t tiles_per_stream,
                                                            uint32_t *__restrict__ esc_cnt) {
  __shared__ uint32_t smem[8];
  const int64_t base = (int64_t)blockIdx.x * tiles_per_stream;
  uint32_t carry = 0;
  for (uint32_t t0 = 0; t0 < tiles_per_stream; t0 += kBlock) {
    const uint32_t t = t0 + threadIdx.x;
    const uint32_t v = t < tiles_per_stream ? tile_cnt[base + t] : 0u;
    uint32_t total;
    const uint32_t ex = block_exclusive_scan(v, smem, &total);
    if (t < tiles_per_stream) tile_off[base + t] = carry + ex;
    carry += total;
  }
  if (esc_cnt && threadIdx.x == 0) esc_cnt[blockIdx.x] = carry;
}

// esc_off = exclusive prefix sum of esc_cnt over all streams (one workgroup).
__global__ __launch_bounds__(kBlock) void scan_streams_kernel(const uint32_t *__restrict__ esc_cnt,
                                                              uint64_t *__restrict__ esc_off, int64_t n_streams,
                                                              uint64_t esc_cap, uint32_t *status) {
  __shared__ uint32_t smem[8];
  uint64_t carry = 0;
  for (int64_t s0 = 0; s0 < n_streams; s0 += kBlock) {
    const int64_t s = s0 + threadIdx.x;
    const uint32_t v = s < n_streams ? esc_cnt[s] : 0u;  // a block of 256 streams holds < 2^32 escapes
    uint32_t total;
    const uint32_t ex = block_exclusive_scan(v, smem, &total);
    if (s < n_streams) esc_off[s] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0 && carry > esc_cap) raise(status, PLC_ERR_CAPACITY);
}

// One wavefront gathers the escapes of one tile again from its symbols and the actual values, 64 chunks at
// a time, and writes them from dst on; for a tile whose staging row overflowed, or that has none.
__device__ __forceinline__ void regather_tile(const CodecArgs &a, uint16_t *__restrict__ esc_vals, uint64_t esc_cap,
                                              uint32_t stream, uint32_t tile, uint64_t dst, int lane) {
  for (int round = 0; round < kBlock / 64; ++round) {
    const Coord q = locate_chunk(a, stream, tile, (uint32_t)(round * 64 + lane));
    uint2 sv = make_uint2(0u, 0u);
    uint32_t n_esc = 0;
    if (q.valid) {
      sv = *reinterpret_cast<const uint2 *>(a.symbols + q.sym);
#pragma unroll
      for (int e = 0; e < kChunk; ++e) n_esc += (((e < 4 ? sv.x : sv.y) >> (8 * (e & 3))) & 255u) == PLC_ESCAPE;
    }
    uint32_t wave_total;
    uint64_t at = dst + wave_escape_prefix(n_esc, &wave_total);
    if (n_esc) {
      const uint16_t *act = (q.c ? a.act_v : a.act_k) + q.act;
#pragma unroll
      for (int e = 0; e < kChunk; ++e) {
        if ((((e < 4 ? sv.x : sv.y) >> (8 * (e & 3))) & 255u) == PLC_ESCAPE) {
          if (at < esc_cap) esc_vals[at] = act[e];
          ++at;
        }
      }
    }
    dst += wave_total;
  }
}

// Escapes of every tile from the symbols to their place in the stream's list, where no staging rows were
// written (symbols that some other pass produced); one wavefront per tile.
__global__ __launch_bounds__(kBlock) void gather_escapes_kernel(const CodecArgs a, uint16_t *__restrict__ esc_vals,
                                                                uint64_t esc_cap,
                                                                const uint64_t *__restrict__ esc_off,
                                                                int64_t n_tiles) {
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
  if (t >= n_tiles) return;
  if (a.tile_cnt[t] == 0) return;  // uniform per wavefront
  const uint32_t stream = (uint32_t)(t / a.tiles_per_stream);
  const uint32_t tile = (uint32_t)(t - (int64_t)stream * a.tiles_per_stream);
  regather_tile(a, esc_vals, esc_cap, stream, tile, esc_off[stream] + a.tile_off[t], lane);
}

// Move every tile's escapes from its staging row to their place in the stream's list.  A wavefront takes
// 64 tiles in a row, a lane looks up the count and the destination of one of them, and the wavefront then
// copies the rows one after the other (a row holds at most two wavefronts' worth).  A tile that overflowed
// its row is gathered again from the symbols.
__global__ __launch_bounds__(kBlock) void compact_escapes_kernel(const CodecArgs a, uint16_t *__restrict__ esc_vals,
                                                                 uint64_t esc_cap,
                                                                 const uint64_t *__restrict__ esc_off,
                                                                 int64_t n_tiles) {
  const int lane = threadIdx.x & 63;
  const int64_t t0 = ((int64_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6)) * 64;
  if (t0 >= n_tiles) return;
  const int64_t t = t0 + lane;
  uint32_t cnt = 0, stream = 0;
  uint64_t dst = 0;
  if (t < n_tiles) {
    cnt = a.tile_cnt[t];
    if (cnt) {
      stream = (uint32_t)(t / a.tiles_per_stream);
      dst = esc_off[stream] + a.tile_off[t];
    }
  }
  uint64_t todo = __ballot(cnt != 0);
  while (todo) {  // uniform
    const int j = __builtin_ctzll(todo);
    todo &= todo - 1;
    const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)cnt, j);
    const uint64_t d = (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)dst, j) |
                       (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(dst >> 32), j) << 32;
    if (c <= (uint32_t)kEscStage) {
      const uint16_t *row = a.esc_stage + (t0 + j) * kEscStage;
#pragma unroll
      for (uint32_t i = (uint32_t)lane; i < (uint32_t)kEscStage; i += 64)
        if (i < c && d + i < esc_cap) esc_vals[d + i] = row[i];
    } else {
      const uint32_t s = (uint32_t)__builtin_amdgcn_readlane((int)stream, j);
      regather_tile(a, esc_vals, esc_cap, s, (uint32_t)(t0 + j - (int64_t)s * a.tiles_per_stream), d, lane);
    }
  }
  static_assert(kEscStage == 128, "two passes of a wavefront over a staging row");
}

// ---------------------------------------------------------------------------
// Decode: prediction again, plus the dequantised residual
// ---------------------------------------------------------------------------
template <int K, bool COND>
__global__ __launch_bounds__(kBlock) void reconstruct_kernel(const CodecArgs a) {
  __shared__ uint32_t smem[8];
  const Coord q = locate(a);
  const bool tile_has_escapes = a.tile_cnt[blockIdx.x] != 0;  // uniform
  uint2 sv = make_uint2(0u, 0u);
  half8 out;
  uint32_t n_esc = 0;
  if (q.valid) {
    const uint16_t *cand = (q.c ? a.cand_v : a.cand_k) + q.cand;
    sv = *reinterpret_cast<const uint2 *>(a.symbols + q.sym);
    float pred[kChunk];
    predict_chunk<K, COND>(a, q, cand, pred);
    const float step = COND ? position_step(a, q.row) : a.delta;
    out = add_back8(sv, step, pred, &n_esc);
  }
  if (tile_has_escapes) {
    uint32_t total;
    const uint32_t rank = block_exclusive_scan(n_esc, smem, &total);
    if (n_esc) {
      uint64_t src = a.esc_off[q.stream] + a.tile_off[blockIdx.x] + rank;
      uint16_t raw[kChunk];
#pragma unroll
      for (int e = 0; e < kChunk; ++e) {
        raw[e] = 0;
        if ((((e < 4 ? sv.x : sv.y) >> (8 * (e & 3))) & 255u) == PLC_ESCAPE) {
          if (src < a.esc_len) {
            raw[e] = a.esc_in[src];
          } else {
            raise(a.status, PLC_ERR_CORRUPT);
          }
          ++src;
          out[e] = __builtin_bit_cast(_Float16, raw[e]);
        }
      }
    }
  }
  if (q.valid) {
    uint16_t *dst = (q.c ? a.out_v : a.out_k) + q.act;
    store16_stream(dst, __builtin_bit_cast(uint4, out));
  }
}

// Overwrite the escaped components of a tile's output with their raw values from the stream's list
// (for outputs written by a kernel that does not handle escapes itself); one workgroup per tile.
__global__ __launch_bounds__(kBlock) void patch_escapes_kernel(const CodecArgs a) {
  __shared__ uint32_t smem[8];
  if (a.tile_cnt[blockIdx.x] == 0) return;  // uniform
  const Coord q = locate(a);
  uint2 sv = make_uint2(0u, 0u);
  uint32_t n_esc = 0;
  if (q.valid) {
    sv = *reinterpret_cast<const uint2 *>(a.symbols + q.sym);
#pragma unroll
    for (int e = 0; e < kChunk; ++e) n_esc += (((e < 4 ? sv.x : sv.y) >> (8 * (e & 3))) & 255u) == PLC_ESCAPE;
  }
  uint32_t total;
  const uint32_t rank = block_exclusive_scan(n_esc, smem, &total);
  if (n_esc) {
    uint64_t src = a.esc_off[q.stream] + a.tile_off[blockIdx.x] + rank;
    uint16_t *dst = (q.c ? a.out_v : a.out_k) + q.act;
#pragma unroll
    for (int e = 0; e < kChunk; ++e) {
      if ((((e < 4 ? sv.x : sv.y) >> (8 * (e & 3))) & 255u) == PLC_ESCAPE) {
        if (src < a.esc_len) {
          dst[e] = a.esc_in[src];
        } else {
          raise(a.status, PLC_ERR_CORRUPT);
        }
        ++src;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
struct Plan {
  int64_t n_streams, syms_per_stream, chunks_per_stream, tiles_per_stream, n_tiles, rows;
  size_t off_weights, off_tile_cnt, off_tile_off, off_stage, total;
};

bool make_plan(const plc_dims *dm, Plan *p) {
  if (!dm) return false;
  if (dm->S < 1 || dm->L < 1 || dm->H < 1 || dm->n < 1) return false;
  if (dm->k < 1 || dm->k > 32) return false;
  if (dm->d < kChunk || dm->d % kChunk) return false;
  if (!(dm->delta > 0.0f) || !(dm->delta < 3.0e38f)) return false;
  if (dm->qmax < 1 || dm->qmax > 127) return false;
  for (int a = 0; a < 5; ++a)
    if (dm->cand_stride[a] < 0 || dm->cand_stride[a] % kChunk) return false;
  for (int a = 0; a < 4; ++a)
    if (dm->act_stride[a] < 0 || dm->act_stride[a] % kChunk) return false;
  p->n_streams = (int64_t)dm->S * dm->L * dm->H;
  p->syms_per_stream = 2ll * dm->n * dm->d;
  p->chunks_per_stream = p->syms_per_stream / kChunk;
  p->tiles_per_stream = (p->chunks_per_stream + kBlock - 1) / kBlock;
  p->n_tiles = p->n_streams * p->tiles_per_stream;
  p->rows = (int64_t)dm->S * dm->n;
  if (p->syms_per_stream >= (1ll << 32)) return false;  // u32 counts per stream
  if (p->n_tiles >= (1ll << 31) || p->n_streams >= (1ll << 31)) return false;
  p->off_weights = 0;
  p->off_tile_cnt = align_up((size_t)p->rows * dm->k * sizeof(float), 256);
  p->off_tile_off = p->off_tile_cnt + align_up((size_t)p->n_tiles * sizeof(uint32_t), 256);
  p->off_stage = p->off_tile_off + align_up((size_t)p->n_tiles * sizeof(uint32_t), 256);
  p->total = p->off_stage + align_up((size_t)p->n_tiles * kEscStage * sizeof(uint16_t), 256);
  return true;
}

bool aligned(const void *p, size_t a) { return p && (reinterpret_cast<uintptr_t>(p) % a) == 0; }

void fill_args(const plc_dims *dm, const Plan &p, void *ws, CodecArgs *a) {
  char *w = static_cast<char *>(ws);
  a->weights = reinterpret_cast<const float *>(w + p.off_weights);
  a->tile_cnt = reinterpret_cast<uint32_t *>(w + p.off_tile_cnt);
  a->tile_off = reinterpret_cast<const uint32_t *>(w + p.off_tile_off);
  a->esc_stage = reinterpret_cast<uint16_t *>(w + p.off_stage);
  a->L = dm->L;
  a->H = dm->H;
  a->n = dm->n;
  a->k = dm->k;
  a->d8 = dm->d / kChunk;
  a->tiles_per_stream = (uint32_t)p.tiles_per_stream;
  a->chunks_per_stream = (uint32_t)p.chunks_per_stream;
  for (int i = 0; i < 5; ++i) a->cs[i] = dm->cand_stride[i];
  for (int i = 0; i < 4; ++i) a->as[i] = dm->act_stride[i];
  a->syms_per_stream = p.syms_per_stream;
  a->delta = dm->delta;
  a->qmax = (float)dm->qmax;
}

template <template <int> class Launcher>
void dispatch_k(int k, const CodecArgs &a, unsigned grid, hipStream_t st) {
  switch (k) {
#define PLC_CASE(K) \
  case K:           \
    Launcher<K>::run(a, grid, st); \
    break;
    PLC_CASE(1) PLC_CASE(2) PLC_CASE(3) PLC_CASE(4) PLC_CASE(5) PLC_CASE(6) PLC_CASE(7) PLC_CASE(8)
    PLC_CASE(12) PLC_CASE(16) PLC_CASE(20)
#undef PLC_CASE
    default:
      Launcher<0>::run(a, grid, st);
  }
}

// Unused dynamic LDS that caps the workgroups a compute unit holds.  Eight workgroups of the weighted-mean
// kernels keep 8 x 256 x (k + 1) x 16 bytes of loads in flight per compute unit, more than HBM needs at k = 8,
// and the extra only spreads the access stream: with six (24 KB each) the k = 8 kernels measured 2-4 % faster
// (predict 0.842 -> 0.820 ms and 27.8 -> 26.7 ms, reconstruct 0.823 -> 0.788 ms on the Llama-shaped and the
// 64-session configuration), with five or four no better, with three slower.  At k = 4 the prediction pass
// gains from seven (3.95 -> 3.75 ms at 32,768 positions) and the reconstruction from none.
unsigned occupancy_pad(int k, bool encode) {
  if (k >= 8) return 24576u;
  if (k >= 4 && encode) return 21000u;
  return 0u;
}

template <int K>
struct LaunchPredict {
  static void run(const CodecArgs &a, unsigned grid, hipStream_t st) {
    if (a.chosen) {
      hipLaunchKernelGGL(predict_residual_cond_kernel<K>, dim3((grid + kCondTiles - 1) / kCondTiles), dim3(kBlock), 0,
                         st, a, grid);
    } else if (a.counts) {
      const uint32_t T = a.tiles_per_stream > (uint32_t)kHistLongStream ? 2u : 1u;
      const uint32_t pad = a.k >= 4 ? 24576u : 0u;  // measured best for this kernel at k = 4 and k = 8 alike
      const uint32_t wgs = (a.tiles_per_stream + T - 1) / T;
      hipLaunchKernelGGL(predict_residual_hist_kernel<K>, dim3((grid / a.tiles_per_stream) * wgs), dim3(kBlock),
                         pad, st, a, a.counts, wgs, T);
    } else {
      hipLaunchKernelGGL(predict_residual_kernel<K>, dim3(grid), dim3(kBlock), occupancy_pad(a.k, true), st, a);
    }
  }
};
template <int K>
struct LaunchReconstruct {
  static void run(const CodecArgs &a, unsigned grid, hipStream_t st) {
    if (a.chosen) {
      hipLaunchKernelGGL((reconstruct_kernel<K, true>), dim3(grid), dim3(kBlock), 0, st, a);
    } else {
      hipLaunchKernelGGL((reconstruct_kernel<K, false>), dim3(grid), dim3(kBlock), occupancy_pad(a.k, false), st, a);
    }
  }
};

// Nearest candidate of every position by the key row of layer 0, head 0; one thread per position.
__global__ __launch_bounds__(kBlock) void select_candidate_kernel(const uint16_t *__restrict__ cand_k,
                                                                  const uint16_t *__restrict__ act_k, int64_t rows,
                                                                  int n, int k, int d, int64_t cs_s, int64_t cs_i,
                                                                  int64_t cs_j, int64_t as_s, int64_t as_i,
                                                                  float limit, int32_t *__restrict__ chosen) {
  const int64_t row = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (row >= rows) return;
  const int64_t s = row / n, i = row - s * n;
  const _Float16 *act = reinterpret_cast<const _Float16 *>(act_k) + s * as_s + i * as_i;
  const _Float16 *cand = reinterpret_cast<const _Float16 *>(cand_k) + s * cs_s + i * cs_i;
  int best_j = -1;
  float best = 0.0f;
  for (int j = 0; j < k; ++j) {
    const _Float16 *c = cand + j * cs_j;
    float acc = 0.0f;
    for (int e = 0; e < d; ++e) {
      const float diff = (float)act[e] - (float)c[e];
      acc = __builtin_fmaf(diff, diff, acc);
    }
    if (best_j < 0 ? (acc == acc) : (acc < best)) {
      best_j = j;
      best = acc;
    }
  }
  if (best_j >= 0 && !(best <= limit)) best_j = -1;
  chosen[row] = best_j;
}

}  // namespace
}  // namespace plc

using namespace plc;

extern "C" size_t plc_workspace_bytes(const plc_dims *dims) {
  Plan p;
  return make_plan(dims, &p) ? p.total : 0;
}

namespace plc {
namespace {

int encode_floats(const plc_dims *dims, const void *cand_k, const void *cand_v, const float *probs,
                  const int32_t *chosen, const uint8_t *bits, float range, int trace_id, const void *act_k, const void *act_v, uint8_t *symbols,
                  uint16_t *esc_vals, uint64_t esc_cap, uint32_t *esc_cnt, uint64_t *esc_off, float *pred_out,
                  void *ws, size_t ws_bytes, uint32_t *status, void *stream, uint32_t *counts = nullptr) {
  Plan p;
  if (!make_plan(dims, &p)) return PLC_ERR_INVALID;
  if (!aligned(cand_k, 16) || !aligned(cand_v, 16) || !aligned(act_k, 16) || !aligned(act_v, 16))
    return PLC_ERR_INVALID;
  if (!aligned(symbols, 8) || !aligned(probs, 4) || !aligned(esc_cnt, 4) || !aligned(esc_off, 8))
    return PLC_ERR_INVALID;
  if (!aligned(status, 4) || !aligned(ws, 256) || ws_bytes < p.total) return PLC_ERR_INVALID;
  if (pred_out && !aligned(pred_out, 16)) return PLC_ERR_INVALID;
  if (esc_cap > 0 && !aligned(esc_vals, 2)) return PLC_ERR_INVALID;
  hipStream_t st = static_cast<hipStream_t>(stream);

  CodecArgs a = {};
  fill_args(dims, p, ws, &a);
  a.cand_k = static_cast<const uint16_t *>(cand_k);
  a.cand_v = static_cast<const uint16_t *>(cand_v);
  a.act_k = static_cast<const uint16_t *>(act_k);
  a.act_v = static_cast<const uint16_t *>(act_v);
  a.symbols = symbols;
  a.pred_out = pred_out;
  a.status = status;
  a.chosen = chosen;
  a.bits = bits;
  a.range = range;
  a.counts = counts;
  float *weights = const_cast<float *>(a.weights);
  uint32_t *tile_off = const_cast<uint32_t *>(a.tile_off);

  hipLaunchKernelGGL(weights_kernel, dim3((unsigned)((p.rows + kBlock - 1) / kBlock)), dim3(kBlock), 0, st, probs,
                     weights, p.rows, dims->k, status);
  if (counts)
    hipLaunchKernelGGL(zero_counts_kernel, dim3((unsigned)((p.n_streams * 256 + kBlock - 1) / kBlock)), dim3(kBlock), 0,
                       st, counts, p.n_streams * 256);
  {
    TraceScope trace(trace_id, st);
    dispatch_k<LaunchPredict>(dims->k, a, (unsigned)p.n_tiles, st);
  }
  hipLaunchKernelGGL(scan_tiles_kernel, dim3((unsigned)p.n_streams), dim3(kBlock), 0, st, a.tile_cnt, tile_off,
                     (uint32_t)p.tiles_per_stream, esc_cnt);
  hipLaunchKernelGGL(scan_streams_kernel, dim3(1), dim3(kBlock), 0, st, esc_cnt, esc_off, p.n_streams, esc_cap,
                     status);
  hipLaunchKernelGGL(compact_escapes_kernel, dim3((unsigned)((p.n_tiles + kBlock - 1) / kBlock)), dim3(kBlock), 0, st,
                     a, esc_vals, esc_cap, esc_off, p.n_tiles);
  return launch_status();
}

int decode_floats(const plc_dims *dims, const void *cand_k, const void *cand_v, const float *probs,
                  const int32_t *chosen, const uint8_t *bits, float range, int trace_id, const uint8_t *symbols, const uint16_t *esc_vals,
                  uint64_t esc_len, const uint64_t *esc_off, void *out_k, void *out_v, void *ws, size_t ws_bytes,
                  uint32_t *status, void *stream) {
  Plan p;
  if (!make_plan(dims, &p)) return PLC_ERR_INVALID;
  if (!aligned(cand_k, 16) || !aligned(cand_v, 16) || !aligned(out_k, 16) || !aligned(out_v, 16))
    return PLC_ERR_INVALID;
  if (!aligned(symbols, 8) || !aligned(probs, 4) || !aligned(esc_off, 8)) return PLC_ERR_INVALID;
  if (!aligned(status, 4) || !aligned(ws, 256) || ws_bytes < p.total) return PLC_ERR_INVALID;
  if (esc_len > 0 && !aligned(esc_vals, 2)) return PLC_ERR_INVALID;
  hipStream_t st = static_cast<hipStream_t>(stream);

  CodecArgs a = {};
  fill_args(dims, p, ws, &a);
  a.cand_k = static_cast<const uint16_t *>(cand_k);
  a.cand_v = static_cast<const uint16_t *>(cand_v);
  a.out_k = static_cast<uint16_t *>(out_k);
  a.out_v = static_cast<uint16_t *>(out_v);
  a.symbols = const_cast<uint8_t *>(symbols);
  a.esc_in = esc_vals;
  a.esc_len = esc_len;
  a.esc_off = esc_off;
  a.status = status;
  a.chosen = chosen;
  a.bits = bits;
  a.range = range;
  float *weights = const_cast<float *>(a.weights);
  uint32_t *tile_off = const_cast<uint32_t *>(a.tile_off);

  hipLaunchKernelGGL(weights_kernel, dim3((unsigned)((p.rows + kBlock - 1) / kBlock)), dim3(kBlock), 0, st, probs,
                     weights, p.rows, dims->k, status);
  hipLaunchKernelGGL(count_escapes_kernel, dim3((unsigned)((p.n_tiles + kBlock / 64 - 1) / (kBlock / 64))), dim3(kBlock), 0, st,
                     a, (uint32_t)p.n_tiles);
  hipLaunchKernelGGL(scan_tiles_kernel, dim3((unsigned)p.n_streams), dim3(kBlock), 0, st, a.tile_cnt, tile_off,
                     (uint32_t)p.tiles_per_stream, (uint32_t *)nullptr);
  {
    TraceScope trace(trace_id, st);
    dispatch_k<LaunchReconstruct>(dims->k, a, (unsigned)p.n_tiles, st);
  }
  return launch_status();
}

}  // namespace
}  // namespace plc

int plc::gather_escapes(const plc_dims *dims, const void *act_k, const void *act_v, const uint8_t *symbols,
                        uint16_t *esc_vals, uint64_t esc_cap, uint32_t *esc_cnt, uint64_t *esc_off, void *ws,
                        size_t ws_bytes, uint32_t *status, hipStream_t st, bool launch) {
  Plan p;
  if (!make_plan(dims, &p)) return PLC_ERR_INVALID;
  if (!aligned(act_k, 16) || !aligned(act_v, 16) || !aligned(symbols, 8) || !aligned(esc_cnt, 4) ||
      !aligned(esc_off, 8) || !aligned(status, 4) || !aligned(ws, 256) || ws_bytes < p.total)
    return PLC_ERR_INVALID;
  if (esc_cap > 0 && !aligned(esc_vals, 2)) return PLC_ERR_INVALID;
  if (!launch) return PLC_OK;
  CodecArgs a = {};
  fill_args(dims, p, ws, &a);
  a.act_k = static_cast<const uint16_t *>(act_k);
  a.act_v = static_cast<const uint16_t *>(act_v);
  a.symbols = const_cast<uint8_t *>(symbols);
  a.status = status;
  uint32_t *tile_off = const_cast<uint32_t *>(a.tile_off);
  hipLaunchKernelGGL(count_escapes_kernel, dim3((unsigned)((p.n_tiles + kBlock / 64 - 1) / (kBlock / 64))), dim3(kBlock), 0, st,
                     a, (uint32_t)p.n_tiles);
  hipLaunchKernelGGL(scan_tiles_kernel, dim3((unsigned)p.n_streams), dim3(kBlock), 0, st, a.tile_cnt, tile_off,
                     (uint32_t)p.tiles_per_stream, esc_cnt);
  hipLaunchKernelGGL(scan_streams_kernel, dim3(1), dim3(kBlock), 0, st, esc_cnt, esc_off, p.n_streams, esc_cap,
                     status);
  hipLaunchKernelGGL(gather_escapes_kernel, dim3((unsigned)((p.n_tiles + kBlock / 64 - 1) / (kBlock / 64))),
                     dim3(kBlock), 0, st, a, esc_vals, esc_cap, esc_off, p.n_tiles);
  return launch_status();
}

int plc::patch_escapes(const plc_dims *dims, const uint8_t *symbols, const uint16_t *esc_vals, uint64_t esc_len,
                       const uint64_t *esc_off, void *out_k, void *out_v, void *ws, size_t ws_bytes,
                       uint32_t *status, hipStream_t st, bool launch) {
  Plan p;
  if (!make_plan(dims, &p)) return PLC_ERR_INVALID;
  if (!aligned(out_k, 16) || !aligned(out_v, 16) || !aligned(symbols, 8) || !aligned(esc_off, 8) ||
      !aligned(status, 4) || !aligned(ws, 256) || ws_bytes < p.total)
    return PLC_ERR_INVALID;
  if (esc_len > 0 && !aligned(esc_vals, 2)) return PLC_ERR_INVALID;
  if (!launch) return PLC_OK;
  CodecArgs a = {};
  fill_args(dims, p, ws, &a);
  a.out_k = static_cast<uint16_t *>(out_k);
  a.out_v = static_cast<uint16_t *>(out_v);
  a.symbols = const_cast<uint8_t *>(symbols);
  a.esc_in = esc_vals;
  a.esc_len = esc_len;
  a.esc_off = esc_off;
  a.status = status;
  uint32_t *tile_off = const_cast<uint32_t *>(a.tile_off);
  hipLaunchKernelGGL(count_escapes_kernel, dim3((unsigned)((p.n_tiles + kBlock / 64 - 1) / (kBlock / 64))), dim3(kBlock), 0, st,
                     a, (uint32_t)p.n_tiles);
  hipLaunchKernelGGL(scan_tiles_kernel, dim3((unsigned)p.n_streams), dim3(kBlock), 0, st, a.tile_cnt, tile_off,
                     (uint32_t)p.tiles_per_stream, (uint32_t *)nullptr);
  hipLaunchKernelGGL(patch_escapes_kernel, dim3((unsigned)p.n_tiles), dim3(kBlock), 0, st, a);
  return launch_status();
}

extern "C" int plc_predict_residual(const plc_dims *dims, const void *cand_k, const void *cand_v,
                                    const float *probs, const void *act_k, const void *act_v,
                                    uint8_t *symbols, uint16_t *esc_vals, uint64_t esc_cap,
                                    uint32_t *esc_cnt, uint64_t *esc_off, float *pred_out, void *ws,
                                    size_t ws_bytes, uint32_t *status, void *stream) {
  return encode_floats(dims, cand_k, cand_v, probs, nullptr, nullptr, 0.0f, PLC_TRACE_PREDICT, act_k, act_v, symbols, esc_vals,
                       esc_cap, esc_cnt, esc_off, pred_out, ws, ws_bytes, status, stream);
}

// ---------------------------------------------------------------------------
// plc_predict_residual for callers that cannot allocate: the workspace is a buffer of the library's own
// ---------------------------------------------------------------------------
// Device memory that lives in the library's code object, one copy per GPU, held until the process ends.
// Host code never uses the array's name as an address: the address on a device is looked up once, with
// that device current, and kept.
static __device__ __align__(256) unsigned char scratch[PLC_STATIC_SCRATCH_BYTES];

namespace plc {
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void *g_scratch_ptr[kMaxDevices] = {};

// The current device's copy of `scratch`, or null if the runtime cannot name it.
void *static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}
}  // namespace
}  // namespace plc

extern "C" int plc_predict_residual_hist(const plc_dims *dims, const void *cand_k, const void *cand_v,
                                         const float *probs, const void *act_k, const void *act_v,
                                         uint8_t *symbols, uint16_t *esc_vals, uint64_t esc_cap,
                                         uint32_t *esc_cnt, uint64_t *esc_off, float *pred_out, uint32_t *counts,
                                         void *ws, size_t ws_bytes, uint32_t *status, void *stream) {
  if (!aligned(counts, 4)) return PLC_ERR_INVALID;
  return encode_floats(dims, cand_k, cand_v, probs, nullptr, nullptr, 0.0f, PLC_TRACE_PREDICT, act_k, act_v, symbols, esc_vals,
                       esc_cap, esc_cnt, esc_off, pred_out, ws, ws_bytes, status, stream, counts);
}

extern "C" int plc_predict_residual_noalloc(const plc_dims *dims, const void *cand_k, const void *cand_v,
                                            const float *probs, const void *act_k, const void *act_v,
                                            uint8_t *symbols, uint16_t *esc_vals, uint64_t esc_cap,
                                            uint32_t *esc_cnt, uint64_t *esc_off, float *pred_out,
                                            uint32_t *status, void *stream) {
  Plan p;
  if (!make_plan(dims, &p)) return PLC_ERR_INVALID;
  if (p.total > (size_t)PLC_STATIC_SCRATCH_BYTES) return PLC_ERR_SCRATCH;
  void *ws = static_scratch();
  if (!ws) return PLC_ERR_HIP;
  // Every word of the workspace that a kernel reads has been written earlier in the same call (weights,
  // per-tile counts, their prefix sums, the staged escapes up to each tile's count), so nothing of the
  // previous call's contents needs clearing.
  return encode_floats(dims, cand_k, cand_v, probs, nullptr, nullptr, 0.0f, PLC_TRACE_PREDICT, act_k, act_v, symbols,
                       esc_vals, esc_cap, esc_cnt, esc_off, pred_out, ws, p.total, status, stream);
}

extern "C" int plc_predict_residual_cond(const plc_dims *dims, const void *cand_k, const void *cand_v,
                                         const float *probs, const int32_t *chosen, const void *act_k,
                                         const void *act_v, uint8_t *symbols, uint16_t *esc_vals,
                                         uint64_t esc_cap, uint32_t *esc_cnt, uint64_t *esc_off, float *pred_out,
                                         void *ws, size_t ws_bytes, uint32_t *status, void *stream) {
  if (!aligned(chosen, 4)) return PLC_ERR_INVALID;
  return encode_floats(dims, cand_k, cand_v, probs, chosen, nullptr, 0.0f, PLC_TRACE_PREDICT_COND, act_k, act_v, symbols,
                       esc_vals, esc_cap, esc_cnt, esc_off, pred_out, ws, ws_bytes, status, stream);
}

extern "C" int plc_reconstruct(const plc_dims *dims, const void *cand_k, const void *cand_v, const float *probs,
                               const uint8_t *symbols, const uint16_t *esc_vals, uint64_t esc_len,
                               const uint64_t *esc_off, void *out_k, void *out_v, void *ws, size_t ws_bytes,
                               uint32_t *status, void *stream) {
  return decode_floats(dims, cand_k, cand_v, probs, nullptr, nullptr, 0.0f, PLC_TRACE_RECONSTRUCT, symbols, esc_vals, esc_len,
                       esc_off, out_k, out_v, ws, ws_bytes, status, stream);
}

namespace plc {
namespace {

// plc_rans_decode_reconstruct (chosen = null), plc_rans_decode_reconstruct_cond and, with bits and n_tables
// tables per stream, plc_rans_decode_reconstruct_adapt
int decode_and_reconstruct(const plc_dims *dims, const uint16_t *freq, const uint32_t *states,
                           const uint16_t *words, uint64_t words_len, const uint64_t *word_off,
                           const uint32_t *n_words, int32_t chunk_syms, const void *cand_k, const void *cand_v,
                           const float *probs, const int32_t *chosen, const uint8_t *bits, float range,
                           int32_t n_tables, const uint16_t *esc_vals, uint64_t esc_len,
                           const uint64_t *esc_off, uint8_t *symbols, void *out_k, void *out_v, void *ws,
                           size_t ws_bytes, uint32_t *status, void *stream) {
  Plan p;
  if (!make_plan(dims, &p)) return PLC_ERR_INVALID;
  // the checks of plc_reconstruct first, so that a refusal leaves nothing enqueued
  if (!aligned(cand_k, 16) || !aligned(cand_v, 16) || !aligned(out_k, 16) || !aligned(out_v, 16))
    return PLC_ERR_INVALID;
  if (!aligned(symbols, 8) || !aligned(probs, 4) || !aligned(esc_off, 8)) return PLC_ERR_INVALID;
  if (!aligned(status, 4) || !aligned(ws, 256) || ws_bytes < p.total) return PLC_ERR_INVALID;
  if (esc_len > 0 && !aligned(esc_vals, 2)) return PLC_ERR_INVALID;
  if (chunk_syms != 0 ||
      !decode_fused_supported(p.n_streams, p.syms_per_stream, dims->k, chosen != nullptr, bits != nullptr)) {
    const int rc = bits ? plc_rans_decode_bucketed(freq, states, words, words_len, word_off, n_words, p.n_streams,
                                                   p.syms_per_stream, chunk_syms, 2 * dims->d, dims->L * dims->H,
                                                   bits, n_tables, symbols, status, stream)
                        : plc_rans_decode(freq, states, words, words_len, word_off, n_words, p.n_streams,
                                          p.syms_per_stream, chunk_syms, symbols, status, stream);
    if (rc) return rc;
    return decode_floats(dims, cand_k, cand_v, probs, chosen, bits, range,
                         chosen ? PLC_TRACE_RECONSTRUCT_COND : PLC_TRACE_RECONSTRUCT, symbols, esc_vals, esc_len,
                         esc_off, out_k, out_v, ws, ws_bytes, status, stream);
  }
  hipStream_t st = static_cast<hipStream_t>(stream);

  CodecArgs a = {};
  fill_args(dims, p, ws, &a);
  a.out_k = static_cast<uint16_t *>(out_k);
  a.out_v = static_cast<uint16_t *>(out_v);
  a.symbols = symbols;
  a.esc_in = esc_vals;
  a.esc_len = esc_len;
  a.esc_off = esc_off;
  a.status = status;
  ReconView r = {};
  r.cand_k = static_cast<const uint16_t *>(cand_k);
  r.cand_v = static_cast<const uint16_t *>(cand_v);
  r.out_k = a.out_k;
  r.out_v = a.out_v;
  r.weights = a.weights;
  r.chosen = chosen;
  r.bits = bits;
  r.range = range;
  for (int i = 0; i < 5; ++i) r.cs[i] = a.cs[i];
  for (int i = 0; i < 4; ++i) r.as[i] = a.as[i];
  r.L = a.L, r.H = a.H, r.n = a.n, r.k = a.k, r.d8 = a.d8;
  r.delta = a.delta;
  r.esc_in = esc_vals;
  r.esc_len = esc_len;
  r.esc_off = esc_off;

  const int rc = rans_decode_fused(freq, states, words, words_len, word_off, n_words, p.n_streams,
                                   p.syms_per_stream, n_tables, symbols, r, status, st, false);
  if (rc) return rc;  // nothing enqueued
  hipLaunchKernelGGL(weights_kernel, dim3((unsigned)((p.rows + kBlock - 1) / kBlock)), dim3(kBlock), 0, st, probs,
                     const_cast<float *>(a.weights), p.rows, dims->k, status);
  return rans_decode_fused(freq, states, words, words_len, word_off, n_words, p.n_streams, p.syms_per_stream,
                           n_tables, symbols, r, status, st, true);
}

}  // namespace
}  // namespace plc

extern "C" int plc_rans_decode_reconstruct(const plc_dims *dims, const uint16_t *freq, const uint32_t *states,
                                           const uint16_t *words, uint64_t words_len, const uint64_t *word_off,
                                           const uint32_t *n_words, int32_t chunk_syms, const void *cand_k,
                                           const void *cand_v, const float *probs, const uint16_t *esc_vals,
                                           uint64_t esc_len, const uint64_t *esc_off, uint8_t *symbols,
                                           void *out_k, void *out_v, void *ws, size_t ws_bytes, uint32_t *status,
                                           void *stream) {
  return decode_and_reconstruct(dims, freq, states, words, words_len, word_off, n_words, chunk_syms, cand_k, cand_v,
                                probs, nullptr, nullptr, 0.0f, 0, esc_vals, esc_len, esc_off, symbols, out_k, out_v,
                                ws, ws_bytes, status, stream);
}

extern "C" int plc_rans_decode_reconstruct_cond(const plc_dims *dims, const uint16_t *freq, const uint32_t *states,
                                                const uint16_t *words, uint64_t words_len,
                                                const uint64_t *word_off, const uint32_t *n_words,
                                                int32_t chunk_syms, const void *cand_k, const void *cand_v,
                                                const float *probs, const int32_t *chosen,
                                                const uint16_t *esc_vals, uint64_t esc_len, const uint64_t *esc_off,
                                                uint8_t *symbols, void *out_k, void *out_v, void *ws,
                                                size_t ws_bytes, uint32_t *status, void *stream) {
  if (!aligned(chosen, 4)) return PLC_ERR_INVALID;
  return decode_and_reconstruct(dims, freq, states, words, words_len, word_off, n_words, chunk_syms, cand_k, cand_v,
                                probs, chosen, nullptr, 0.0f, 0, esc_vals, esc_len, esc_off, symbols, out_k, out_v,
                                ws, ws_bytes, status, stream);
}

extern "C" int plc_rans_decode_reconstruct_adapt(const plc_dims *dims, const uint16_t *freq, const uint32_t *states,
                                                 const uint16_t *words, uint64_t words_len,
                                                 const uint64_t *word_off, const uint32_t *n_words,
                                                 int32_t chunk_syms, int32_t n_tables, const void *cand_k,
                                                 const void *cand_v, const float *probs, const int32_t *chosen,
                                                 const uint8_t *bits, float range, const uint16_t *esc_vals,
                                                 uint64_t esc_len, const uint64_t *esc_off, uint8_t *symbols,
                                                 void *out_k, void *out_v, void *ws, size_t ws_bytes,
                                                 uint32_t *status, void *stream) {
  if (!aligned(chosen, 4) || !bits || !(range > 0.0f) || !(range < 3.0e38f)) return PLC_ERR_INVALID;
  if (n_tables < 1 || n_tables > PLC_MAX_BITS) return PLC_ERR_INVALID;
  return decode_and_reconstruct(dims, freq, states, words, words_len, word_off, n_words, chunk_syms, cand_k, cand_v,
                                probs, chosen, bits, range, n_tables, esc_vals, esc_len, esc_off, symbols, out_k,
                                out_v, ws, ws_bytes, status, stream);
}

extern "C" int plc_reconstruct_cond(const plc_dims *dims, const void *cand_k, const void *cand_v,
                                    const float *probs, const int32_t *chosen, const uint8_t *symbols,
                                    const uint16_t *esc_vals, uint64_t esc_len, const uint64_t *esc_off,
                                    void *out_k, void *out_v, void *ws, size_t ws_bytes, uint32_t *status,
                                    void *stream) {
  if (!aligned(chosen, 4)) return PLC_ERR_INVALID;
  return decode_floats(dims, cand_k, cand_v, probs, chosen, nullptr, 0.0f, PLC_TRACE_RECONSTRUCT_COND, symbols, esc_vals,
                       esc_len, esc_off, out_k, out_v, ws, ws_bytes, status, stream);
}

extern "C" int plc_predict_residual_adapt(const plc_dims *dims, const void *cand_k, const void *cand_v,
                                          const float *probs, const int32_t *chosen, const uint8_t *bits,
                                          float range, const void *act_k, const void *act_v, uint8_t *symbols,
                                          uint16_t *esc_vals, uint64_t esc_cap, uint32_t *esc_cnt,
                                          uint64_t *esc_off, float *pred_out, void *ws, size_t ws_bytes,
                                          uint32_t *status, void *stream) {
  if (!aligned(chosen, 4) || !bits || !(range > 0.0f) || !(range < 3.0e38f)) return PLC_ERR_INVALID;
  return encode_floats(dims, cand_k, cand_v, probs, chosen, bits, range, PLC_TRACE_PREDICT_COND, act_k, act_v,
                       symbols, esc_vals, esc_cap, esc_cnt, esc_off, pred_out, ws, ws_bytes, status, stream);
}

extern "C" int plc_reconstruct_adapt(const plc_dims *dims, const void *cand_k, const void *cand_v,
                                     const float *probs, const int32_t *chosen, const uint8_t *bits, float range,
                                     const uint8_t *symbols, const uint16_t *esc_vals, uint64_t esc_len,
                                     const uint64_t *esc_off, void *out_k, void *out_v, void *ws, size_t ws_bytes,
                                     uint32_t *status, void *stream) {
  if (!aligned(chosen, 4) || !bits || !(range > 0.0f) || !(range < 3.0e38f)) return PLC_ERR_INVALID;
  return decode_floats(dims, cand_k, cand_v, probs, chosen, bits, range, PLC_TRACE_RECONSTRUCT_COND, symbols,
                       esc_vals, esc_len, esc_off, out_k, out_v, ws, ws_bytes, status, stream);
}

extern "C" int plc_select_candidate(const plc_dims *dims, const void *cand_k, const void *act_k,
                                    float max_mean_sq, int32_t *chosen, void *stream) {
  Plan p;
  if (!make_plan(dims, &p)) return PLC_ERR_INVALID;
  if (!aligned(cand_k, 16) || !aligned(act_k, 16) || !aligned(chosen, 4)) return PLC_ERR_INVALID;
  if (!(max_mean_sq >= 0.0f)) return PLC_ERR_INVALID;
  hipLaunchKernelGGL(select_candidate_kernel, dim3((unsigned)((p.rows + kBlock - 1) / kBlock)), dim3(kBlock), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint16_t *>(cand_k),
                     static_cast<const uint16_t *>(act_k), p.rows, dims->n, dims->k, dims->d, dims->cand_stride[0],
                     dims->cand_stride[3], dims->cand_stride[4], dims->act_stride[0], dims->act_stride[3],
                     max_mean_sq * (float)dims->d, chosen);
  return launch_status();
}
