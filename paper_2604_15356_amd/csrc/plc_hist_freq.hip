// Symbol statistics for the entropy coder: per-stream histograms (LDS atomics)
// and the integer frequency tables on the 2^12 scale.  Definitions are in
// include/plc.h.
#include "plc_device.h"

namespace plc {
namespace {

constexpr int kHistSegment = 64 * 1024;  // symbols per workgroup

__global__ __launch_bounds__(kBlock) void zero_u32_kernel(uint32_t *p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// Each workgroup counts one segment of one stream into LDS histograms, then adds the non-empty bins to
// the stream's global counts.  Lanes that hit the same counter in one instruction are served one after
// the other, and quantised residuals crowd into a few symbols (a dozen on the token-conditional path),
// so every wavefront has kHistCopies histograms, a lane using copy lane mod kHistCopies; the copies
// start 8 banks apart, so that equal symbols in different copies do not share a bank either.
constexpr int kHistCopies = 8;
constexpr int kHistStride = 256 + 8;

__global__ __launch_bounds__(kBlock) void histogram_kernel(const uint8_t *__restrict__ symbols,
                                                           int64_t syms_per_stream, uint32_t segs_per_stream,
                                                           uint32_t *__restrict__ counts) {
  __shared__ uint32_t hist[kBlock / 64][kHistCopies][kHistStride];
  const uint32_t stream = blockIdx.x / segs_per_stream;
  const uint32_t seg = blockIdx.x - stream * segs_per_stream;
  const int wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < (kBlock / 64) * kHistCopies * kHistStride; i += kBlock) (&hist[0][0][0])[i] = 0u;
  __syncthreads();
  uint32_t *mine = hist[wave][threadIdx.x & (kHistCopies - 1)];

  const int64_t seg_begin = (int64_t)seg * kHistSegment;
  const int64_t seg_end = seg_begin + kHistSegment < syms_per_stream ? seg_begin + kHistSegment : syms_per_stream;
  const uint8_t *base = symbols + (int64_t)stream * syms_per_stream;
  const uint8_t *p = base + seg_begin;
  const uint8_t *end = base + seg_end;
  // bytes before the first 16-byte boundary
  const uintptr_t mis = reinterpret_cast<uintptr_t>(p) & 15u;
  int64_t head = mis ? 16 - (int64_t)mis : 0;
  if (head > end - p) head = end - p;
  if ((int64_t)threadIdx.x < head) atomicAdd(&mine[p[threadIdx.x]], 1u);
  p += head;
  const int64_t n_vec = (end - p) / 16;
  const uint4 *pv = reinterpret_cast<const uint4 *>(p);
  for (int64_t i = threadIdx.x; i < n_vec; i += kBlock) {
    const uint4 v = load16_stream(pv + i);
    const uint32_t wds[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
      for (int b = 0; b < 4; ++b) atomicAdd(&mine[(wds[j] >> (8 * b)) & 255u], 1u);
    }
  }
  p += n_vec * 16;
  if ((int64_t)threadIdx.x < end - p) atomicAdd(&mine[p[threadIdx.x]], 1u);
  __syncthreads();

  uint32_t c = 0;
#pragma unroll
  for (int w = 0; w < kBlock / 64; ++w)
#pragma unroll
    for (int r = 0; r < kHistCopies; ++r) c += hist[w][r][threadIdx.x];
  if (c) atomicAdd(&counts[(int64_t)stream * 256 + threadIdx.x], c);
}

// The same with one histogram per bit depth: the depth of a symbol is that of its position, and a
// thread's 16 symbols always share a position (positions hold a multiple of 16 symbols).
__global__ __launch_bounds__(kBlock) void histogram_bucketed_kernel(const uint8_t *__restrict__ symbols,
                                                                    int64_t syms_per_stream, uint32_t segs_per_stream,
                                                                    uint32_t syms_per_pos, uint32_t streams_per_session,
                                                                    const uint8_t *__restrict__ bits, int n_tables,
                                                                    uint32_t pos_lanes, uint32_t *__restrict__ counts,
                                                                    uint32_t *status) {
  __shared__ uint32_t hist[kBlock / 64][PLC_MAX_BITS][256];
  const uint32_t stream = blockIdx.x / segs_per_stream;
  const uint32_t seg = blockIdx.x - stream * segs_per_stream;
  const int wave = threadIdx.x >> 6;
#pragma unroll
  for (int w = 0; w < kBlock / 64; ++w)
#pragma unroll
    for (int t = 0; t < PLC_MAX_BITS; ++t) hist[w][t][threadIdx.x] = 0u;
  __syncthreads();

  const int64_t seg_begin = (int64_t)seg * kHistSegment;
  const int64_t seg_end = seg_begin + kHistSegment < syms_per_stream ? seg_begin + kHistSegment : syms_per_stream;
  const uint8_t *base = symbols + (int64_t)stream * syms_per_stream;
  const uint8_t *brow = bits + (int64_t)(stream / streams_per_session) * (syms_per_stream / syms_per_pos);
  for (int64_t t0 = seg_begin + (int64_t)threadIdx.x * 16; t0 < seg_end; t0 += kBlock * 16) {
    int b = brow[t0 / syms_per_pos];
    if (b < 1 || b > n_tables) {
      raise(status, PLC_ERR_INVALID);
      b = 1;
    }
    uint32_t *h = hist[wave][b - 1];
    const uint4 v = load16_stream(base + t0);
    const uint32_t wds[4] = {v.x, v.y, v.z, v.w};
    // At coarse steps most residuals quantise to zero, and every lane would queue at that one counter: the
    // zeros are counted apart and summed over the `pos_lanes` neighbouring lanes that share the position
    // (a power of two, at most 16) before one lane adds them.
    uint32_t zeros = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t sym = (wds[j] >> (8 * q)) & 255u;
        if (sym == kZeroSymbol)
          ++zeros;
        else
          atomicAdd(&h[sym], 1u);
      }
    }
#pragma unroll
    for (uint32_t m = 1; m < 16; m <<= 1)
      if (m < pos_lanes) zeros += __shfl_xor(zeros, (int)m);
    if ((threadIdx.x & (pos_lanes - 1)) == 0 && zeros) atomicAdd(&h[kZeroSymbol], zeros);
  }
  __syncthreads();
  for (int t = 0; t < n_tables; ++t) {
    uint32_t c = 0;
#pragma unroll
    for (int w = 0; w < kBlock / 64; ++w) c += hist[w][t][threadIdx.x];
    if (c) atomicAdd(&counts[((int64_t)stream * n_tables + t) * 256 + threadIdx.x], c);
  }
}

// One wavefront per stream; lane L owns symbols 4L .. 4L+3.  `allow_empty`: a row without any count is
// not an error and gets all-zero frequencies (a bit depth that does not occur in a stream).
__global__ __launch_bounds__(kBlock) void build_freq_kernel(const uint32_t *__restrict__ counts, int64_t n_streams,
                                                            uint16_t *__restrict__ freq, uint16_t *__restrict__ cum,
                                                            bool allow_empty, uint32_t *status) {
  const int lane = threadIdx.x & 63;
  const int64_t stream = (int64_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
  if (stream >= n_streams) return;  // uniform per wavefront
  const uint4 cv = *reinterpret_cast<const uint4 *>(counts + stream * 256 + lane * 4);
  const uint32_t cnt[4] = {cv.x, cv.y, cv.z, cv.w};

  // inclusive running counts C (64-bit)
  uint64_t run[4];
  run[0] = cnt[0];
  run[1] = run[0] + cnt[1];
  run[2] = run[1] + cnt[2];
  run[3] = run[2] + cnt[3];
  uint64_t inc = run[3];
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint64_t up = __shfl_up(inc, off, 64);
    if (lane >= off) inc += up;
  }
  const uint64_t before = inc - run[3];
  const uint64_t T = __shfl(inc, 63, 64);
  if (T == 0) {
    if (lane == 0 && !allow_empty) raise(status, PLC_ERR_INVALID);
    *reinterpret_cast<uint2 *>(freq + stream * 256 + lane * 4) = make_uint2(0u, 0u);
    if (cum) {
      for (int r = 0; r < 4; ++r) cum[stream * 257 + lane * 4 + r] = 0;
      if (lane == 63) cum[stream * 257 + 256] = 0;
    }
    return;
  }
  // f[s] = floor(C[s] * 4096 / T) - floor(C[s-1] * 4096 / T)
  uint32_t f[4];
  uint64_t prev = (before * PLC_RANS_SCALE) / T;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const uint64_t cur = ((before + run[r]) * PLC_RANS_SCALE) / T;
    f[r] = (uint32_t)(cur - prev);
    prev = cur;
  }
  // symbols that occur but were scaled to zero, in ascending symbol order
  uint64_t need[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) need[r] = __ballot(cnt[r] > 0 && f[r] == 0);
  if (need[0] | need[1] | need[2] | need[3]) {
    for (int s = 0; s < 256; ++s) {
      const int r = s & 3, owner = s >> 2;
      if (!((need[r] >> owner) & 1ull)) continue;  // uniform
      // donor: largest current frequency, lowest symbol on ties
      uint32_t best = 0;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const uint32_t key = (f[t] << 8) | (255u - (uint32_t)(lane * 4 + t));
        best = key > best ? key : best;
      }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) {
        const uint32_t o = __shfl_xor(best, off, 64);
        best = o > best ? o : best;
      }
      const int donor = 255 - (int)(best & 255u);
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        if (lane * 4 + t == donor) f[t] -= 1;
        if (lane * 4 + t == s) f[t] = 1;
      }
    }
  }
  *reinterpret_cast<uint2 *>(freq + stream * 256 + lane * 4) = make_uint2(f[0] | (f[1] << 16), f[2] | (f[3] << 16));
  if (cum) {
    uint32_t lane_sum = f[0] + f[1] + f[2] + f[3];
    uint32_t incf = lane_sum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t up = __shfl_up(incf, off, 64);
      if (lane >= off) incf += up;
    }
    uint32_t acc = incf - lane_sum;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      cum[stream * 257 + lane * 4 + r] = (uint16_t)acc;
      acc += f[r];
    }
    if (lane == 63) cum[stream * 257 + 256] = (uint16_t)acc;
  }
}

}  // namespace
}  // namespace plc

using namespace plc;

extern "C" int plc_histogram(const uint8_t *symbols, int64_t n_streams, int64_t syms_per_stream, uint32_t *counts,
                             void *stream) {
  if (!symbols || !counts || n_streams < 1 || syms_per_stream < 1) return PLC_ERR_INVALID;
  if (syms_per_stream >= (1ll << 32)) return PLC_ERR_INVALID;
  if (reinterpret_cast<uintptr_t>(counts) % 16) return PLC_ERR_INVALID;
  const int64_t segs = (syms_per_stream + kHistSegment - 1) / kHistSegment;
  if (n_streams * segs >= (1ll << 31) || n_streams >= (1ll << 31) / 256) return PLC_ERR_INVALID;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int64_t n = n_streams * 256;
  hipLaunchKernelGGL(zero_u32_kernel, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, st, counts, n);
  {
    TraceScope trace(PLC_TRACE_HISTOGRAM, st);
    hipLaunchKernelGGL(histogram_kernel, dim3((unsigned)(n_streams * segs)), dim3(kBlock), 0, st, symbols,
                       syms_per_stream, (uint32_t)segs, counts);
  }
  return launch_status();
}

extern "C" int plc_build_freq(const uint32_t *counts, int64_t n_streams, uint16_t *freq, uint16_t *cum,
                              uint32_t *status, void *stream) {
  if (!counts || !freq || !status || n_streams < 1) return PLC_ERR_INVALID;
  if (reinterpret_cast<uintptr_t>(counts) % 16 || reinterpret_cast<uintptr_t>(freq) % 8) return PLC_ERR_INVALID;
  if (cum && reinterpret_cast<uintptr_t>(cum) % 2) return PLC_ERR_INVALID;
  const int64_t blocks = (n_streams + kBlock / 64 - 1) / (kBlock / 64);
  if (blocks >= (1ll << 31)) return PLC_ERR_INVALID;
  hipLaunchKernelGGL(build_freq_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, static_cast<hipStream_t>(stream),
                     counts, n_streams, freq, cum, false, status);
  return launch_status();
}

extern "C" int plc_histogram_bucketed(const uint8_t *symbols, int64_t n_streams, int64_t syms_per_stream,
                                      int32_t syms_per_pos, int32_t streams_per_session, const uint8_t *bits,
                                      int32_t n_tables, uint32_t *counts, uint32_t *status, void *stream) {
  if (!symbols || !counts || !bits || !status || n_streams < 1 || syms_per_stream < 1) return PLC_ERR_INVALID;
  if (syms_per_stream >= (1ll << 32) || n_tables < 1 || n_tables > PLC_MAX_BITS) return PLC_ERR_INVALID;
  if (syms_per_pos < 32 || syms_per_pos % 32 || syms_per_stream % syms_per_pos || streams_per_session < 1)
    return PLC_ERR_INVALID;
  if (reinterpret_cast<uintptr_t>(counts) % 16 || reinterpret_cast<uintptr_t>(symbols) % 16) return PLC_ERR_INVALID;
  const int64_t segs = (syms_per_stream + kHistSegment - 1) / kHistSegment;
  if (n_streams * segs >= (1ll << 31) || n_streams >= (1ll << 31) / (256 * PLC_MAX_BITS)) return PLC_ERR_INVALID;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int64_t n = n_streams * n_tables * 256;
  // neighbouring lanes (16 symbols each) that always share a position: a power of two dividing syms_per_pos / 16
  uint32_t pos_lanes = 2;
  while (pos_lanes < 16 && (syms_per_pos / 16) % (2 * pos_lanes) == 0) pos_lanes *= 2;
  hipLaunchKernelGGL(zero_u32_kernel, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, st, counts, n);
  hipLaunchKernelGGL(histogram_bucketed_kernel, dim3((unsigned)(n_streams * segs)), dim3(kBlock), 0, st, symbols,
                     syms_per_stream, (uint32_t)segs, (uint32_t)syms_per_pos, (uint32_t)streams_per_session, bits,
                     n_tables, pos_lanes, counts, status);
  return launch_status();
}

extern "C" int plc_build_freq_bucketed(const uint32_t *counts, int64_t n_streams, int32_t n_tables, uint16_t *freq,
                                       uint32_t *status, void *stream) {
  if (!counts || !freq || !status || n_streams < 1 || n_tables < 1 || n_tables > PLC_MAX_BITS) return PLC_ERR_INVALID;
  if (reinterpret_cast<uintptr_t>(counts) % 16 || reinterpret_cast<uintptr_t>(freq) % 8) return PLC_ERR_INVALID;
  const int64_t rows = n_streams * n_tables;
  const int64_t blocks = (rows + kBlock / 64 - 1) / (kBlock / 64);
  if (blocks >= (1ll << 31)) return PLC_ERR_INVALID;
  hipLaunchKernelGGL(build_freq_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, static_cast<hipStream_t>(stream),
                     counts, rows, freq, (uint16_t *)nullptr, true, status);
  return launch_status();
}
