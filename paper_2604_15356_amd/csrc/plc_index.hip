// The index stream of token-conditional coding: which of the k candidates the true token was (or
// that it was none of them), one symbol per position, coded under the model's own probabilities so
// that a position costs about the token's surprisal (Thm. "Sequential entropy bound", Sec. 4.2).
// See include/plc.h for the format.
//
// The stream is tiny next to the residuals (one symbol per position against 2*L*H*d of them), but with
// one session it is a single chain of n / 32 steps, so the per-position tables are prepared off the
// chain; words go straight to global memory at positions ranked from the emission mask.
#include <cmath>

#include "plc_device.h"

namespace plc {
namespace {

constexpr int kLanes = PLC_RANS_LANES;
constexpr uint32_t kScale = PLC_RANS_SCALE;
constexpr uint32_t kLow = 1u << 16;
constexpr int kMaxK = 32;

// Frequencies of the k + 1 index symbols of one probability row; returns false for an invalid row
// (its negative / NaN entries are taken as 0, so the table is usable either way).
__device__ bool index_table(const float *__restrict__ p, int k, uint32_t f[kMaxK + 1]) {
  bool ok = true;
  float c = 0.0f;
  uint32_t prev = 0;
  for (int j = 0; j < k; ++j) {
    float pj = p[j];
    if (!(pj >= 0.0f)) {
      ok = false;
      pj = 0.0f;
    }
    c = c + pj;
    float scaled = __builtin_floorf(c * 4096.0f);
    if (!(scaled < 4096.0f)) scaled = 4096.0f;  // probability above one (or an overflow) is clipped
    const uint32_t b = (uint32_t)scaled;
    f[j] = b - prev;
    prev = b;
  }
  f[k] = kScale - prev;
  for (int j = 0; j <= k; ++j) {
    if (f[j] == 0) {
      int donor = 0;
      for (int m = 1; m <= k; ++m)
        if (f[m] > f[donor]) donor = m;
      f[donor] -= 1;
      f[j] = 1;
    }
  }
  return ok;
}

// Both coders give a session one workgroup of four wavefronts.  The chain of rANS steps is sequential,
// but what a step needs from its position -- the table made from that position's probabilities -- is not:
// wavefronts 1-3 prepare the tables of the next six groups (192 positions, one per thread, the table living
// in the thread's own LDS row) while wavefront 0 codes the current six from LDS; one barrier per tile.
constexpr int kTileGroups = 6;
constexpr int kTilePos = kTileGroups * kLanes;  // 192 = the three helper wavefronts
constexpr int kRow = kMaxK + 2;                 // k + 1 frequencies or k + 2 cumulative values, padded
constexpr int kIdxStageWords = 8192;            // decoder: index streams up to this many words are read from LDS

// Frequencies of one row into an LDS row (same arithmetic as index_table).
__device__ __forceinline__ bool index_table_lds(const float *__restrict__ p, int k, uint16_t *f) {
  bool ok = true;
  float c = 0.0f;
  uint32_t prev = 0;
  for (int j = 0; j < k; ++j) {
    float pj = p[j];
    if (!(pj >= 0.0f)) {
      ok = false;
      pj = 0.0f;
    }
    c = c + pj;
    float scaled = __builtin_floorf(c * 4096.0f);
    if (!(scaled < 4096.0f)) scaled = 4096.0f;
    const uint32_t b = (uint32_t)scaled;
    f[j] = (uint16_t)(b - prev);
    prev = b;
  }
  f[k] = (uint16_t)(kScale - prev);
  for (int j = 0; j <= k; ++j) {
    if (f[j] == 0) {
      int donor = 0;
      for (int m = 1; m <= k; ++m)
        if (f[m] > f[donor]) donor = m;
      f[donor] -= 1;
      f[j] = 1;
    }
  }
  return ok;
}

__global__ __launch_bounds__(256) void index_encode_kernel(const float *__restrict__ probs,
                                                           const int32_t *__restrict__ chosen, int n, int k,
                                                           uint32_t *__restrict__ states, uint16_t *__restrict__ words,
                                                           const uint64_t *__restrict__ word_off, uint64_t word_cap,
                                                           uint32_t *__restrict__ n_words, uint32_t *status) {
  __shared__ uint16_t rows[kTilePos][kRow];
  __shared__ uint32_t pair[2][kTileGroups][kLanes];  // f | cum << 16 of the symbol to code
  const int s = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint16_t *out = words + word_off[s];
  uint32_t x = kLow;
  uint64_t nw = 0;  // uniform
  const int groups = (n + kLanes - 1) / kLanes;
  const int tiles = (groups + kTileGroups - 1) / kTileGroups;
  // tile t holds groups top(t) - 1 down to top(t) - 6, top(t) = groups - 6 t (the encoder walks downwards)
  for (int it = 0; it <= tiles; ++it) {
    if (wave > 0) {
      if (it < tiles) {
        const int u = threadIdx.x - 64, gi = u >> 5, l = u & 31;
        const int g = groups - kTileGroups * it - 1 - gi;
        const int i = g * kLanes + l;
        uint32_t v = 1u;  // f = 1, cum = 0 for lanes without a symbol (never used)
        if (g >= 0 && i < n) {
          const int64_t row = (int64_t)s * n + i;
          if (!index_table_lds(probs + row * k, k, rows[u])) raise(status, PLC_ERR_INVALID);
          int j = chosen[row];
          if (j < -1 || j >= k) {
            raise(status, PLC_ERR_INVALID);
            j = -1;
          }
          const int sym = j < 0 ? k : j;
          uint32_t cs = 0;
          for (int m = 0; m < sym; ++m) cs += rows[u][m];
          v = (uint32_t)rows[u][sym] | (cs << 16);
        }
        pair[it & 1][gi][l] = v;
      }
    } else if (it > 0) {
      const int t = it - 1;
      for (int gi = 0; gi < kTileGroups; ++gi) {
        const int g = groups - kTileGroups * t - 1 - gi;
        if (g < 0) break;  // uniform
        const int i = g * kLanes + lane;
        const bool has = lane < kLanes && i < n;
        const uint32_t v = pair[t & 1][gi][lane & 31];
        const uint32_t fs = v & 0xffffu, cs = v >> 16;
        // The sequential definition visits lane 31 first: a lane's word comes after those of the
        // emitting lanes above it.
        const bool emit = has && (x >> 20) >= fs;
        const uint32_t mask = (uint32_t)__ballot(emit);
        if (emit) {
          const uint32_t above = lane == 31 ? 0u : mask >> (lane + 1);
          const uint64_t pos = nw + (uint32_t)__builtin_popcount(above);
          if (pos < word_cap) {
            out[pos] = (uint16_t)(x & 0xffffu);
          } else {
            raise(status, PLC_ERR_CAPACITY);
          }
          x >>= 16;
        }
        nw += (uint32_t)__builtin_popcount(mask);
        if (has) x = (x / fs) * kScale + (x % fs) + cs;
      }
    }
    __syncthreads();
  }
  if (wave == 0) {
    if (lane < kLanes) states[(int64_t)s * kLanes + lane] = x;
    if (lane == 0) n_words[s] = (uint32_t)(nw < word_cap ? nw : word_cap);
  }
}

__global__ __launch_bounds__(256) void index_decode_kernel(const float *__restrict__ probs,
                                                           const uint32_t *__restrict__ states,
                                                           const uint16_t *__restrict__ words, uint64_t words_len,
                                                           const uint64_t *__restrict__ word_off,
                                                           const uint32_t *__restrict__ n_words, int n, int k,
                                                           int32_t *__restrict__ chosen, uint32_t *status) {
  // cumulative frequencies cum[0..k+1] of every position of a tile (rows of 68 bytes, read as words)
  __shared__ __attribute__((aligned(4))) uint16_t cums[2][kTilePos][kRow];
  __shared__ uint16_t wstage[kIdxStageWords];
  const int s = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bool rans_lane = lane < kLanes;
  const uint64_t base = word_off[s];
  uint64_t ptr = n_words[s];  // uniform
  bool corrupt = base > words_len || ptr > words_len - base;
  if (corrupt) ptr = 0;
  // A session's index stream is short (a few bits per position): it is copied to LDS first, so that a
  // renormalising lane does not wait for HBM inside the chain of steps.  A longer one is read in place.
  const bool staged = ptr <= (uint64_t)kIdxStageWords;  // uniform
  if (staged)
    for (uint32_t i = threadIdx.x; i < (uint32_t)ptr; i += 256) wstage[i] = words[base + i];
  uint32_t x = rans_lane ? states[(int64_t)s * kLanes + lane] : kLow;
  const int groups = (n + kLanes - 1) / kLanes;
  const int tiles = (groups + kTileGroups - 1) / kTileGroups;
  __syncthreads();
  for (int it = 0; it <= tiles; ++it) {
    if (wave > 0) {
      if (it < tiles) {
        const int u = threadIdx.x - 64;
        const int i = (kTileGroups * it + (u >> 5)) * kLanes + (u & 31);
        if (i < n) {
          uint16_t *row = cums[it & 1][u];
          if (!index_table_lds(probs + ((int64_t)s * n + i) * k, k, row)) raise(status, PLC_ERR_INVALID);
          uint32_t acc = 0;
          for (int m = 0; m <= k; ++m) {  // frequencies -> exclusive prefix sums, in place
            const uint32_t f = row[m];
            row[m] = (uint16_t)acc;
            acc += f;
          }
          row[k + 1] = (uint16_t)acc;  // 4096
        }
      }
    } else if (it > 0) {
      const int t = it - 1;
      for (int gi = 0; gi < kTileGroups; ++gi) {
        const int g = kTileGroups * t + gi;
        if (g >= groups) break;  // uniform
        const int i = g * kLanes + lane;
        const bool has = rans_lane && i < n;
        if (has) {
          const uint16_t *row = cums[t & 1][gi * kLanes + lane];
          const uint32_t slot = x & (kScale - 1);
          int sym = 0;
          uint32_t cs, fs;
          if (k <= 8) {  // uniform
            // the row's ten values in one LDS round trip, then the search in registers: the symbol is the
            // number of interval starts cum[1..k] at or below the slot, its start the largest value at
            // or below the slot and its end the smallest above (cum[k+1] = 4096 always is)
            const uint32_t *r32 = reinterpret_cast<const uint32_t *>(row);
            const uint32_t v[5] = {r32[0], r32[1], r32[2], r32[3], r32[4]};
            cs = 0;
            uint32_t next = kScale;
#pragma unroll
            for (int m = 1; m <= 9; ++m) {
              const uint32_t c = (m & 1) ? v[m >> 1] >> 16 : v[m >> 1] & 0xffffu;
              const bool in = m <= k + 1;  // uniform
              if (in && c <= slot) {
                cs = c > cs ? c : cs;
                sym += m <= k;
              }
              if (in && c > slot) next = c < next ? c : next;
            }
            fs = next - cs;
          } else {
            while (sym < k && row[sym + 1] <= slot) ++sym;  // the symbol whose interval holds the slot
            cs = row[sym];
            fs = (uint32_t)row[sym + 1] - cs;
          }
          chosen[(int64_t)s * n + i] = sym == k ? -1 : sym;
          x = fs * (x >> 12) + slot - cs;
        }
        // Reading lanes are served from the end of the list, lane 0 first.
        const bool need = has && x < kLow;
        const uint32_t mask = (uint32_t)__ballot(need);
        if (need) {
          const uint32_t below = mask & ((1u << lane) - 1u);
          const uint64_t rank = (uint32_t)__builtin_popcount(below);
          uint32_t word = 0;
          if (rank < ptr) {
            word = staged ? wstage[ptr - 1 - rank] : words[base + ptr - 1 - rank];
          } else {
            corrupt = true;
          }
          x = (x << 16) | word;
        }
        const uint32_t used = (uint32_t)__builtin_popcount(mask);
        ptr = used < ptr ? ptr - used : 0;
      }
    }
    __syncthreads();
  }
  if (wave == 0) {
    if (ptr != 0 || (rans_lane && x != kLow)) corrupt = true;
    if (corrupt) raise(status, PLC_ERR_CORRUPT);
  }
}

struct Thresholds {
  uint16_t thr[PLC_MAX_BITS + 1];
};

// Bit depth of every position from the frequency of its index symbol; one thread per position.
__global__ __launch_bounds__(kBlock) void surprisal_bits_kernel(const float *__restrict__ probs,
                                                                const int32_t *__restrict__ chosen, int64_t rows,
                                                                int k, Thresholds t, int bmax,
                                                                uint8_t *__restrict__ bits, uint32_t *status) {
  const int64_t row = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (row >= rows) return;
  uint32_t f[kMaxK + 1];
  if (!index_table(probs + row * k, k, f)) raise(status, PLC_ERR_INVALID);
  int j = chosen[row];
  if (j < -1 || j >= k) {
    raise(status, PLC_ERR_INVALID);
    j = -1;
  }
  const uint32_t fs = f[j < 0 ? k : j];
  int b = 1;
  for (int m = 2; m <= bmax; ++m)
    if (fs <= t.thr[m]) b = m;
  bits[row] = (uint8_t)b;
}

int check(const float *probs, int32_t S, int32_t n, int32_t k, const void *states, const void *word_off,
          const void *n_words, const void *chosen, const void *status) {
  if (S < 1 || n < 1 || k < 1 || k > kMaxK) return PLC_ERR_INVALID;
  if (!probs || !states || !word_off || !n_words || !chosen || !status) return PLC_ERR_INVALID;
  if (reinterpret_cast<uintptr_t>(probs) % 4 || reinterpret_cast<uintptr_t>(states) % 4 ||
      reinterpret_cast<uintptr_t>(word_off) % 8 || reinterpret_cast<uintptr_t>(n_words) % 4 ||
      reinterpret_cast<uintptr_t>(chosen) % 4 || reinterpret_cast<uintptr_t>(status) % 4)
    return PLC_ERR_INVALID;
  return PLC_OK;
}

}  // namespace
}  // namespace plc

using namespace plc;

extern "C" int plc_index_encode(const float *probs, const int32_t *chosen, int32_t S, int32_t n, int32_t k,
                                uint32_t *states, uint16_t *words, const uint64_t *word_off, uint64_t word_cap,
                                uint32_t *n_words, uint32_t *status, void *stream) {
  const int rc = check(probs, S, n, k, states, word_off, n_words, chosen, status);
  if (rc) return rc;
  if ((word_cap > 0 && !words) || reinterpret_cast<uintptr_t>(words) % 2) return PLC_ERR_INVALID;
  hipLaunchKernelGGL(index_encode_kernel, dim3((unsigned)S), dim3(256), 0, static_cast<hipStream_t>(stream), probs,
                     chosen, n, k, states, words, word_off, word_cap, n_words, status);
  return launch_status();
}

extern "C" int plc_index_decode(const float *probs, const uint32_t *states, const uint16_t *words,
                                uint64_t words_len, const uint64_t *word_off, const uint32_t *n_words, int32_t S,
                                int32_t n, int32_t k, int32_t *chosen, uint32_t *status, void *stream) {
  const int rc = check(probs, S, n, k, states, word_off, n_words, chosen, status);
  if (rc) return rc;
  if ((words_len > 0 && !words) || reinterpret_cast<uintptr_t>(words) % 2) return PLC_ERR_INVALID;
  hipLaunchKernelGGL(index_decode_kernel, dim3((unsigned)S), dim3(256), 0, static_cast<hipStream_t>(stream), probs,
                     states, words, words_len, word_off, n_words, n, k, chosen, status);
  return launch_status();
}

extern "C" int plc_surprisal_thresholds(double b0, double hbar, int32_t bmax, uint16_t *thr) {
  if (!(b0 > 0.0) || !(hbar > 0.0) || !(b0 < 1e300) || !(hbar < 1e300)) return PLC_ERR_INVALID;
  if (bmax < 1 || bmax > PLC_MAX_BITS || !thr) return PLC_ERR_INVALID;
  thr[0] = thr[1] = 0;
  for (int m = 2; m <= bmax; ++m) {
    // 4096 * 2^(-m * hbar / b0): the power of two scales the exponential exactly
    const double t = std::floor(std::ldexp(std::exp2(-((double)m * hbar) / b0), 12 /* log2 of the probability scale */));
    thr[m] = (uint16_t)(t < 0.0 ? 0.0 : t > 4096.0 ? 4096.0 : t);
  }
  return PLC_OK;
}

extern "C" int plc_surprisal_bits(const float *probs, const int32_t *chosen, int32_t S, int32_t n, int32_t k,
                                  const uint16_t *thr, int32_t bmax, uint8_t *bits, uint32_t *status,
                                  void *stream) {
  if (S < 1 || n < 1 || k < 1 || k > kMaxK || bmax < 1 || bmax > PLC_MAX_BITS) return PLC_ERR_INVALID;
  if (!probs || !chosen || !thr || !bits || !status) return PLC_ERR_INVALID;
  if (reinterpret_cast<uintptr_t>(probs) % 4 || reinterpret_cast<uintptr_t>(chosen) % 4 ||
      reinterpret_cast<uintptr_t>(status) % 4)
    return PLC_ERR_INVALID;
  Thresholds t = {};
  for (int m = 2; m <= bmax; ++m) {
    if (m > 2 && thr[m] > thr[m - 1]) return PLC_ERR_INVALID;
    t.thr[m] = thr[m];
  }
  const int64_t rows = (int64_t)S * n;
  hipLaunchKernelGGL(surprisal_bits_kernel, dim3((unsigned)((rows + kBlock - 1) / kBlock)), dim3(kBlock), 0,
                     static_cast<hipStream_t>(stream), probs, chosen, rows, k, t, bmax, bits, status);
  return launch_status();
}
