// 32-lane interleaved rANS encoder and decoder.  The bitstream is defined in
// include/plc.h.  The paper only asks for "standard source coding" of the
// residuals (proof of Prop. "Layer orthogonality", Sec. 6.1); interleaved rANS
// is the choice made here because its 32 lanes map onto half a wavefront.
//
// Mapping: one 64-lane wavefront codes two units, lanes 0-31 one unit and
// lanes 32-63 the next.  The 32 lanes of a unit advance in lock step, one
// symbol group (32 symbols) per iteration; positions in the word list come
// from a ballot and a population count, so no atomics are involved and the
// output is deterministic.  The work per unit is a chain of dependent integer
// steps, N/32 long, so these kernels are bound by instruction latency and by
// how many units are in flight, not by HBM.
#include "plc_device.h"

namespace plc {
namespace {

constexpr int kLanes = PLC_RANS_LANES;
constexpr int kScaleBits = 12;
constexpr uint32_t kScale = PLC_RANS_SCALE;
constexpr uint32_t kLow = 1u << 16;
constexpr int kBatch = 16;  // symbol groups between two refills of the staging buffers

struct RansArgs {
  const uint8_t *sym_in;  // encode
  uint8_t *sym_out;       // decode
  const uint16_t *freq;
  uint32_t *states_out;      // encode
  const uint32_t *states_in; // decode
  uint16_t *words_out;       // encode
  const uint16_t *words_in;  // decode
  uint64_t words_len;        // decode
  const uint64_t *word_off;
  uint64_t word_cap;         // encode
  uint32_t *n_words_out;     // encode
  const uint32_t *n_words_in;// decode
  uint32_t *status;
  int64_t n_units, units_per_stream, syms_per_stream, unit_syms;
};

struct Unit {
  bool live;
  int64_t unit, stream, begin;
  uint32_t len;  // symbols in this unit
};

__device__ __forceinline__ Unit locate_unit(const RansArgs &a, int half) {
  Unit u;
  u.unit = (int64_t)blockIdx.x * 2 + half;
  u.live = u.unit < a.n_units;
  const int64_t un = u.live ? u.unit : 0;
  u.stream = un / a.units_per_stream;
  const int64_t chunk = un - u.stream * a.units_per_stream;
  u.begin = chunk * a.unit_syms;
  const int64_t rest = a.syms_per_stream - u.begin;
  u.len = (uint32_t)(rest < a.unit_syms ? rest : a.unit_syms);
  u.unit = un;
  return u;
}

// Lane l of a half-wavefront gets the frequencies of symbols 8l .. 8l+7 and the
// cumulative frequency in front of them.  Returns the table's total.
__device__ __forceinline__ uint32_t load_freq8(const uint16_t *freq, int l, uint32_t f[8], uint32_t *cum0) {
  const uint4 fv = *reinterpret_cast<const uint4 *>(freq + l * 8);
  const uint32_t w[4] = {fv.x, fv.y, fv.z, fv.w};
  uint32_t sum = 0;
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    f[r] = (w[r >> 1] >> (16 * (r & 1))) & 0xffffu;
    sum += f[r];
  }
  uint32_t inc = sum;
#pragma unroll
  for (int off = 1; off < kLanes; off <<= 1) {
    const uint32_t up = __shfl_up(inc, off, kLanes);
    if (l >= off) inc += up;
  }
  *cum0 = inc - sum;
  return __shfl(inc, kLanes - 1, kLanes);
}

__device__ __forceinline__ uint32_t half_mask(uint64_t ballot, int half) {
  return half ? (uint32_t)(ballot >> 32) : (uint32_t)ballot;
}

// ---------------------------------------------------------------------------
// Encoder
// ---------------------------------------------------------------------------
// Table entry per symbol: .x = multiplier for the division by f, .y packs
// f (13 bits) | cum (12 bits) << 13 | sh1 << 25 | sh2 << 26.  The quotient
// floor(x / f) is exact for every 32-bit x (round-up multiplier of width 33,
// applied as  t = mulhi(m, x);  q = (t + ((x - t) >> sh1)) >> sh2).
__device__ __forceinline__ uint2 make_enc_entry(uint32_t f, uint32_t cum) {
  if (f == 0) return make_uint2(0u, 0u);
  const uint32_t l = f > 1 ? 32u - (uint32_t)__builtin_clz(f - 1) : 0u;  // ceil(log2 f)
  const uint64_t num = (uint64_t)((1u << l) - f) << 32;
  const uint32_t m = (uint32_t)(num / f) + 1u;
  const uint32_t sh1 = l < 1 ? l : 1u, sh2 = l > 1 ? l - 1u : 0u;
  return make_uint2(m, f | ((cum & 4095u) << 13) | (sh1 << 25) | (sh2 << 26));
}

__global__ __launch_bounds__(64) void rans_encode_kernel(const RansArgs a) {
  __shared__ uint2 table[2][256];
  const int lane = threadIdx.x, half = lane >> 5, l = lane & 31;
  const Unit u = locate_unit(a, half);

  {
    uint32_t f[8], cum;
    const uint32_t total = load_freq8(a.freq + u.stream * 256, l, f, &cum);
    if (u.live && total != kScale && l == 0) raise(a.status, PLC_ERR_INVALID);
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      table[half][l * 8 + r] = make_enc_entry(f[r], cum);
      cum += f[r];
    }
  }
  __syncthreads();

  const uint8_t *sp = a.sym_in + u.stream * a.syms_per_stream + u.begin;
  uint16_t *wp = a.words_out + (u.live ? a.word_off[u.unit] : 0);
  const int32_t G = u.live ? (int32_t)((u.len + kLanes - 1) / kLanes) : 0;
  const int32_t n_batches = (int32_t)(((a.unit_syms + kLanes - 1) / kLanes + kBatch - 1) / kBatch);
  uint32_t x = kLow;
  uint64_t nw = 0;
  bool zero_freq = false;

  // symbols of the first batch (groups G-1 down to G-16)
  uint32_t nxt[kBatch];
#pragma unroll
  for (int j = 0; j < kBatch; ++j) {
    const int32_t g = G - 1 - j;
    const int64_t t = (int64_t)g * kLanes + l;
    nxt[j] = (g >= 0 && t < (int64_t)u.len) ? sp[t] : 0u;
  }
  for (int32_t b = 0; b < n_batches; ++b) {
    uint32_t cur[kBatch];
#pragma unroll
    for (int j = 0; j < kBatch; ++j) cur[j] = nxt[j];
    // fetch the next batch while this one is coded
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      const int32_t g = G - 1 - (b + 1) * kBatch - j;
      const int64_t t = (int64_t)g * kLanes + l;
      nxt[j] = (g >= 0 && t < (int64_t)u.len) ? sp[t] : 0u;
    }
    uint2 ent[kBatch];
#pragma unroll
    for (int j = 0; j < kBatch; ++j) ent[j] = table[half][cur[j]];
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      const int32_t g = G - 1 - b * kBatch - j;
      const bool active = g >= 0 && (int64_t)g * kLanes + l < (int64_t)u.len;
      const uint32_t fs = ent[j].y & 0x1fffu;
      const uint32_t cs = (ent[j].y >> 13) & 0xfffu;
      const uint32_t sh1 = (ent[j].y >> 25) & 1u, sh2 = ent[j].y >> 26;
      if (active && fs == 0) zero_freq = true;
      // renormalise: x >= f * 2^20, tested on the high bits (f * 2^20 overflows for f = 4096)
      const bool emit = active && (x >> 20) >= fs;
      const uint32_t m32 = half_mask(__ballot(emit), half);
      if (emit) {
        // the encoder visits lane 31 first, so a lane's slot counts the emitting lanes above it
        const uint64_t idx = nw + (uint32_t)__popc((m32 >> l) >> 1);
        if (idx < a.word_cap) wp[idx] = (uint16_t)(x & 0xffffu);
        x >>= 16;
      }
      nw += (uint32_t)__popc(m32);
      if (active) {
        const uint32_t t1 = __umulhi(ent[j].x, x);
        const uint32_t q = (t1 + ((x - t1) >> sh1)) >> sh2;  // floor(x / f)
        x = q * (kScale - fs) + x + cs;                      // q * 4096 + x mod f + cum
      }
    }
  }
  if (u.live) {
    a.states_out[u.unit * kLanes + l] = x;
    if (l == 0) {
      a.n_words_out[u.unit] = (uint32_t)(nw < 0xffffffffull ? nw : 0xffffffffull);
      if (nw > a.word_cap) raise(a.status, PLC_ERR_CAPACITY);
    }
    if (zero_freq) raise(a.status, PLC_ERR_INVALID);
  }
}

// ---------------------------------------------------------------------------
// Decoder
// ---------------------------------------------------------------------------
// Slot table: for each of the 4096 slots, sym | (f - 1) << 8 | (slot - cum) << 20.
// Words are consumed from the end of the unit's list; they are staged through
// an LDS ring of four 512-word blocks (aligned in absolute address), refilled
// one block per batch of 16 groups, which can consume at most 512 words.
constexpr int kRingWords = 2048, kBlockWords = 512;

__device__ __forceinline__ bool load_block(const uint16_t *aligned_base, int32_t blk, int32_t lo, int32_t hi, int l,
                                           uint4 v[2]) {
  bool any = false;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int32_t first = blk * kBlockWords + (2 * l + p) * 8;  // eight words per 16-byte piece
    v[p] = make_uint4(0u, 0u, 0u, 0u);
    if (blk >= 0 && hi > lo && first + 8 > lo && first < hi) {  // piece holds a word of this unit
      v[p] = *reinterpret_cast<const uint4 *>(aligned_base + first);
      any = true;
    }
  }
  return any;
}

__device__ __forceinline__ void store_block(uint16_t *ring, int32_t blk, int l, const uint4 v[2]) {
  uint4 *dst = reinterpret_cast<uint4 *>(ring + ((blk * kBlockWords) & (kRingWords - 1)));
  dst[2 * l] = v[0];
  dst[2 * l + 1] = v[1];
}

__global__ __launch_bounds__(64) void rans_decode_kernel(const RansArgs a) {
  __shared__ uint32_t lut[2][kScale];
  __shared__ __attribute__((aligned(16))) uint16_t ring[2][kRingWords];
  __shared__ uint32_t fc[2][256];  // f | cum << 16
  const int lane = threadIdx.x, half = lane >> 5, l = lane & 31;
  Unit u = locate_unit(a, half);
  bool bad = false;

  // ---- slot table
  {
    uint32_t f[8], cum;
    const uint32_t total = load_freq8(a.freq + u.stream * 256, l, f, &cum);
    if (total != kScale) {  // not a table: decode nothing for this unit
      if (u.live) bad = true;
      u.live = false;
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      fc[half][l * 8 + r] = f[r] | (cum << 16);
      cum += f[r];
    }
  }
  __syncthreads();
  if (u.live) {
    for (int s = 0; s < 256; ++s) {
      const uint32_t e = fc[half][s];
      const uint32_t f = e & 0xffffu, c = e >> 16;
      for (uint32_t o = l; o < f; o += kLanes) lut[half][c + o] = (uint32_t)s | ((f - 1u) << 8) | (o << 20);
    }
  }

  // ---- word list geometry, relative to a 1 KiB-aligned address at or below the unit's first word
  const uint64_t off = u.live ? a.word_off[u.unit] : 0;
  uint32_t n = u.live ? a.n_words_in[u.unit] : 0;
  if (u.live && (off > a.words_len || (uint64_t)n > a.words_len - off)) {
    bad = true;
    u.live = false;
    n = 0;
  }
  const uintptr_t first_addr = reinterpret_cast<uintptr_t>(a.words_in + off);
  const uintptr_t base_addr = first_addr & ~(uintptr_t)(kBlockWords * 2 - 1);
  const uint16_t *aligned_base = reinterpret_cast<const uint16_t *>(base_addr);
  const int32_t lo = (int32_t)((first_addr - base_addr) >> 1);
  const int32_t hi = lo + (int32_t)n;  // n < 2^31 - 512 is checked on the host through syms_per_stream
  int32_t ptr = hi;
  int32_t lowest = ((hi - 1) >> 9) + 1;  // lowest block already staged (none yet)
  {
    uint4 v[2];
    for (int r = 0; r < 2; ++r) {  // the two top blocks
      const int32_t blk = lowest - 1;
      load_block(aligned_base, blk, lo, hi, l, v);
      store_block(ring[half], blk, l, v);
      lowest = blk;
    }
  }
  __syncthreads();

  uint32_t x = u.live ? a.states_in[u.unit * kLanes + l] : kLow;
  uint8_t *sp = a.sym_out + u.stream * a.syms_per_stream + u.begin;
  const int32_t n_batches = (int32_t)(((a.unit_syms + kLanes - 1) / kLanes + kBatch - 1) / kBatch);

  for (int32_t b = 0; b < n_batches; ++b) {
    // stage one more block below if the coming batches may reach it
    const int32_t top = (ptr - 1) >> 9;
    uint4 pre[2];
    const bool fetch = lowest > top - 2;
    const int32_t blk = lowest - 1;
    if (fetch) load_block(aligned_base, blk, lo, hi, l, pre);

#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      const int64_t t = ((int64_t)b * kBatch + j) * kLanes + l;
      const bool active = u.live && t < (int64_t)u.len;
      const uint32_t slot = x & (kScale - 1);
      const uint32_t e = lut[half][slot];
      if (active) {
        x = ((e >> 8) & 0xfffu) * (x >> kScaleBits) + (x >> kScaleBits) + (e >> 20);  // f * (x >> 12) + slot - cum
        sp[t] = (uint8_t)(e & 0xffu);
      }
      const bool need = active && x < kLow;
      const uint32_t m32 = half_mask(__ballot(need), half);
      const int32_t cnt = __popc(m32);
      if (need) {
        // the decoder visits lane 0 first: a lane's word is the rank-th from the top
        const int32_t idx = ptr - 1 - __popc(m32 & ((1u << l) - 1u));
        uint32_t w = 0;
        if (idx >= lo) {
          w = ring[half][idx & (kRingWords - 1)];
        } else {
          bad = true;  // ran out of words
        }
        x = (x << 16) | w;
      }
      ptr = ptr - cnt < lo ? lo : ptr - cnt;
    }
    if (fetch) {
      store_block(ring[half], blk, l, pre);
      lowest = blk;
    }
    __syncthreads();
  }
  // integrity: every word consumed, every lane back at the initial state
  if (u.live && (ptr != lo || x != kLow)) bad = true;
  if (bad) raise(a.status, PLC_ERR_CORRUPT);
}

int check_common(int64_t n_streams, int64_t syms_per_stream, int32_t chunk_syms, RansArgs *a) {
  if (n_streams < 1 || syms_per_stream < 1) return PLC_ERR_INVALID;
  if (syms_per_stream >= (1ll << 31) - 1024) return PLC_ERR_INVALID;
  if (chunk_syms < 0 || chunk_syms % kLanes) return PLC_ERR_INVALID;
  a->units_per_stream = plc_units_per_stream(syms_per_stream, chunk_syms);
  a->unit_syms = chunk_syms > 0 ? chunk_syms : syms_per_stream;
  a->n_units = n_streams * a->units_per_stream;
  a->syms_per_stream = syms_per_stream;
  if ((a->n_units + 1) / 2 >= (1ll << 31)) return PLC_ERR_INVALID;
  return PLC_OK;
}

}  // namespace
}  // namespace plc

using namespace plc;

extern "C" int64_t plc_units_per_stream(int64_t syms_per_stream, int32_t chunk_syms) {
  if (chunk_syms <= 0) return 1;
  return (syms_per_stream + chunk_syms - 1) / chunk_syms;
}

extern "C" int plc_rans_encode(const uint8_t *symbols, int64_t n_streams, int64_t syms_per_stream,
                               int32_t chunk_syms, const uint16_t *freq, uint32_t *states, uint16_t *words,
                               const uint64_t *word_off, uint64_t word_cap_per_unit, uint32_t *n_words,
                               uint32_t *status, void *stream) {
  RansArgs a = {};
  int rc = check_common(n_streams, syms_per_stream, chunk_syms, &a);
  if (rc) return rc;
  if (!symbols || !freq || !states || !word_off || !n_words || !status) return PLC_ERR_INVALID;
  if (word_cap_per_unit > 0 && !words) return PLC_ERR_INVALID;
  if (reinterpret_cast<uintptr_t>(freq) % 16 || reinterpret_cast<uintptr_t>(words) % 2) return PLC_ERR_INVALID;
  a.sym_in = symbols;
  a.freq = freq;
  a.states_out = states;
  a.words_out = words;
  a.word_off = word_off;
  a.word_cap = word_cap_per_unit;
  a.n_words_out = n_words;
  a.status = status;
  {
    TraceScope trace(PLC_TRACE_RANS_ENCODE, static_cast<hipStream_t>(stream));
    hipLaunchKernelGGL(rans_encode_kernel, dim3((unsigned)((a.n_units + 1) / 2)), dim3(64), 0,
                       static_cast<hipStream_t>(stream), a);
  }
  return launch_status();
}

extern "C" int plc_rans_decode(const uint16_t *freq, const uint32_t *states, const uint16_t *words,
                               uint64_t words_len, const uint64_t *word_off, const uint32_t *n_words,
                               int64_t n_streams, int64_t syms_per_stream, int32_t chunk_syms, uint8_t *symbols,
                               uint32_t *status, void *stream) {
  RansArgs a = {};
  int rc = check_common(n_streams, syms_per_stream, chunk_syms, &a);
  if (rc) return rc;
  if (!symbols || !freq || !states || !word_off || !n_words || !status) return PLC_ERR_INVALID;
  if (words_len > 0 && !words) return PLC_ERR_INVALID;
  if (reinterpret_cast<uintptr_t>(freq) % 16 || reinterpret_cast<uintptr_t>(words) % 2) return PLC_ERR_INVALID;
  a.sym_out = symbols;
  a.freq = freq;
  a.states_in = states;
  a.words_in = words;
  a.words_len = words_len;
  a.word_off = word_off;
  a.n_words_in = n_words;
  a.status = status;
  {
    TraceScope trace(PLC_TRACE_RANS_DECODE, static_cast<hipStream_t>(stream));
    hipLaunchKernelGGL(rans_decode_kernel, dim3((unsigned)((a.n_units + 1) / 2)), dim3(64), 0,
                       static_cast<hipStream_t>(stream), a);
  }
  return launch_status();
}
