// Internal helpers shared by the device sources of libplc (not part of the C boundary).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "plc.h"

namespace plc {

// One tile = the 2048 consecutive symbols of a stream that one 256-thread
// workgroup handles: each thread owns one 16-byte chunk of 8 fp16 components.
constexpr int kBlock = 256;
constexpr int kChunk = 8;
constexpr int kTileSyms = kBlock * kChunk;

constexpr uint32_t kZeroSymbol = 127;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));

// 16-byte load of data that is read once: keep it from displacing cache lines that are reused.
__device__ __forceinline__ uint4 load16_stream(const void *p) {
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// Optional event pairs around the main kernel of each call (plc_trace_kernel_events).
struct TraceEvents {
  hipEvent_t start, stop;
};
extern TraceEvents g_trace[PLC_TRACE_COUNT];

struct TraceScope {
  int id;
  hipStream_t st;
  TraceScope(int id_, hipStream_t st_) : id(id_), st(st_) {
    if (g_trace[id].start) (void)hipEventRecord(g_trace[id].start, st);
  }
  ~TraceScope() {
    if (g_trace[id].stop) (void)hipEventRecord(g_trace[id].stop, st);
  }
};

// Stores of data that is written once and not read again by this kernel: non-temporal, so that the
// write stream does not take L2 capacity from the reads (worth 12 % on the predict kernel).
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void store8_stream(void *p, uint32_t a, uint32_t b) {
  const u32x2 v = {a, b};
  __builtin_nontemporal_store(v, reinterpret_cast<u32x2 *>(p));
}
__device__ __forceinline__ void store16_stream(void *p, uint4 a) {
  const u32x4 v = {a.x, a.y, a.z, a.w};
  __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(p));
}

// One candidate's term of a chunk's prediction: pred[e] = fma(w, cand[e], pred[e]) in fp32.
__device__ __forceinline__ void accumulate8(float w, uint4 cv, float pred[kChunk]) {
  const half8 c = __builtin_bit_cast(half8, cv);
#pragma unroll
  for (int e = 0; e < kChunk; ++e) pred[e] = __builtin_fmaf(w, (float)c[e], pred[e]);
}

// Dequantised residual added back to the prediction, for the 8 symbols of a chunk (packed low byte
// first); counts the escapes among them, whose components the caller replaces.
__device__ __forceinline__ half8 add_back8(uint2 sv, float step, const float pred[kChunk], uint32_t *n_esc) {
  half8 out;
#pragma unroll
  for (int e = 0; e < kChunk; ++e) {
    const uint32_t sym = ((e < 4 ? sv.x : sv.y) >> (8 * (e & 3))) & 255u;
    *n_esc += sym == PLC_ESCAPE;
    const float qf = (float)((int)sym - (int)kZeroSymbol);
    float v = __builtin_fmaf(qf, step, pred[e]);
    // Two roundings are the contract: to fp32 here, then to fp16 (nearest even).  Left to itself the
    // compiler may merge both into one fused multiply-add with an fp16 result, which rounds once and
    // lands on the other neighbour when the fp32 value is an exact fp16 tie.
    asm("" : "+v"(v));
    out[e] = (_Float16)v;
  }
  return out;
}

// Number of escapes in the lanes below this one, from the per-lane counts 0..8, by bit planes.
__device__ __forceinline__ uint32_t wave_escape_prefix(uint32_t n_esc, uint32_t *wave_total) {
  uint32_t prefix = 0, total = 0;
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    const uint64_t plane = __ballot((n_esc >> b) & 1u);
    prefix += __builtin_amdgcn_mbcnt_hi((uint32_t)(plane >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)plane, 0u)) << b;
    total += (uint32_t)__builtin_popcountll(plane) << b;
  }
  *wave_total = total;
  return prefix;
}

// What a reconstruction that runs inside the entropy decoder (plc_rans.hip) needs to know; filled in by
// plc_predict.hip, which owns the workspace layout.
struct ReconView {
  const uint16_t *cand_k, *cand_v;
  uint16_t *out_k, *out_v;
  const float *weights;  // [S, n, k] renormalised
  const int32_t *chosen;  // [S, n] index of each position's true candidate or -1; null: always the weighted mean
  const uint8_t *bits;    // [S, n] bit depth of each position (step = range * 2^-bits); null: the step is delta
  float range;
  int64_t cs[5], as[4];  // element strides of the candidates [S,L,H,n,k] and of the output [S,L,H,n]
  int32_t L, H, n, k, d8;
  float delta;
  const uint16_t *esc_in;   // the escape lists, as for plc_reconstruct
  uint64_t esc_len;
  const uint64_t *esc_off;
};
// Whether plc_rans.hip has a decoder that reconstructs as it goes for this many streams and candidates
// (cond: token-conditional prediction; per_depth: with one table per bit depth besides).
bool decode_fused_supported(int64_t n_streams, int64_t syms_per_stream, int k, bool cond, bool per_depth);
// That decoder: plc_rans_decode with one unit per stream, plus out = prediction + symbol * delta for every
// component, escapes from their lists.  With recon.bits: plc_rans_decode_bucketed with n_tables tables per
// stream instead.  The weights must be in place on `st`.  With launch = false the arguments are checked and
// nothing is enqueued.
int rans_decode_fused(const uint16_t *freq, const uint32_t *states, const uint16_t *words, uint64_t words_len,
                      const uint64_t *word_off, const uint32_t *n_words, int64_t n_streams,
                      int64_t syms_per_stream, int32_t n_tables, uint8_t *symbols, const ReconView &recon,
                      uint32_t *status, hipStream_t st, bool launch);

// Escape bookkeeping for callers that produce or consume symbols outside the tile-structured kernels
// (plc_predict.hip): collect the escaped components' raw fp16 values of `act` into the per-stream lists /
// overwrite the escaped components of `out` from the lists.  dims->k and the candidate strides are not used.
// With launch = false the arguments are checked and nothing is enqueued.
int gather_escapes(const plc_dims *dims, const void *act_k, const void *act_v, const uint8_t *symbols,
                   uint16_t *esc_vals, uint64_t esc_cap, uint32_t *esc_cnt, uint64_t *esc_off, void *ws,
                   size_t ws_bytes, uint32_t *status, hipStream_t st, bool launch = true);
int patch_escapes(const plc_dims *dims, const uint8_t *symbols, const uint16_t *esc_vals, uint64_t esc_len,
                  const uint64_t *esc_off, void *out_k, void *out_v, void *ws, size_t ws_bytes, uint32_t *status,
                  hipStream_t st, bool launch = true);

inline int launch_status() { return hipGetLastError() == hipSuccess ? PLC_OK : PLC_ERR_HIP; }

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

__device__ __forceinline__ void raise(uint32_t *status, uint32_t code) {
  if (status) atomicMax(status, code);
}

// Inclusive prefix sum over the 64 lanes of a wavefront.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    uint32_t up = __shfl_up(v, off, 64);
    if (lane >= off) v += up;
  }
  return v;
}

// Exclusive prefix sum of one value per thread over a 256-thread workgroup.
// `smem` needs 5 words.  Returns the exclusive prefix; *total gets the block sum.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *smem, uint32_t *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t inc = wave_inclusive_scan(v);
  __syncthreads();  // protect smem against a previous use
  if (lane == 63) smem[wave] = inc;
  __syncthreads();
  uint32_t base = 0;
#pragma unroll
  for (int w = 0; w < kBlock / 64; ++w) {
    uint32_t s = smem[w];
    if (w < wave) base += s;
  }
  *total = smem[0] + smem[1] + smem[2] + smem[3];
  return base + inc - v;
}

}  // namespace plc
