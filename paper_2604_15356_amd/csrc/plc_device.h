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

// Escape bookkeeping for callers that produce or consume symbols outside the tile-structured kernels
// (plc_predict.hip): collect the escaped components' raw fp16 values of `act` into the per-stream lists /
// overwrite the escaped components of `out` from the lists.  dims->k and the candidate strides are not used.
int gather_escapes(const plc_dims *dims, const void *act_k, const void *act_v, const uint8_t *symbols,
                   uint16_t *esc_vals, uint64_t esc_cap, uint32_t *esc_cnt, uint64_t *esc_off, void *ws,
                   size_t ws_bytes, uint32_t *status, hipStream_t st);
int patch_escapes(const plc_dims *dims, const uint8_t *symbols, const uint16_t *esc_vals, uint64_t esc_len,
                  const uint64_t *esc_off, void *out_k, void *out_v, void *ws, size_t ws_bytes, uint32_t *status,
                  hipStream_t st);

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
