// 32-lane interleaved rANS encoder and decoder.  The bitstream is defined in
// include/plc.h.  The paper only asks for "standard source coding" of the
// residuals (proof of Prop. "Layer orthogonality", Sec. 6.1); interleaved rANS
// is the choice made here because its 32 lanes advance in lock step inside a
// wavefront and the shared word list is addressed with a ballot and a lane
// count, without atomics, so the output is deterministic.
//
// Mapping.  One wavefront codes one unit: lanes 0-31 carry the 32 rANS states
// and lanes 32-63 mirror them exactly (same state, same LDS addresses, same
// values), so that no step needs a lane mask and everything uniform stays in
// scalar registers; all 64 lanes move data between HBM and LDS.  A workgroup holds up to eight
// wavefronts that code consecutive units of the SAME stream and share that
// stream's table in LDS.  Per unit the work is a chain of N/32 dependent
// steps, so the kernels are bound by instruction issue and LDS latency times
// the chain length, and by how many units are in flight -- not by HBM.  The
// inner step is therefore written for a minimal instruction count: symbols,
// words and table entries go through LDS staging buffers that are filled and
// drained 16 groups at a time, and everything uniform stays in scalar
// registers.
#include "plc_device.h"

namespace plc {
namespace {

constexpr int kLanes = PLC_RANS_LANES;
constexpr int kScaleBits = 12;
constexpr uint32_t kScale = PLC_RANS_SCALE;
constexpr uint32_t kLow = 1u << 16;
constexpr int kBatch = 16;                      // symbol groups per staging round
constexpr int kBatchSyms = kBatch * kLanes;     // 512
constexpr int kSuper = 4;                       // encoder: batches fetched per staging round, so that
constexpr int kSuperGroups = kSuper * kBatch;   // the next round's HBM latency hides behind 64 groups
constexpr int kSuperSyms = kSuperGroups * kLanes;
constexpr int kSymStage = kSuperSyms + 32;      // 2048 symbols at any 16-byte misalignment
constexpr int kStagePieces = 3;                 // 16-byte pieces per lane and round (192 >= 130)
constexpr int kMaxWaves = 8;

struct RansArgs {
  const uint8_t *sym_in;       // encode
  uint8_t *sym_out;            // decode
  const uint16_t *freq;
  uint32_t *states_out;        // encode
  const uint32_t *states_in;   // decode
  uint16_t *words_out;         // encode
  const uint16_t *words_in;    // decode
  uint64_t words_len;          // decode
  const uint64_t *word_off;
  uint64_t word_cap;           // encode
  uint32_t *n_words_out;       // encode
  const uint32_t *n_words_in;  // decode
  uint32_t *status;
  int64_t n_units, units_per_stream, syms_per_stream, unit_syms;
  uint32_t wgs_per_stream;
  uint32_t pair_wgs_per_stream;  // rans_encode_pair_kernel with one table: workgroups per stream
  // one table per bit depth (the *_bucketed calls): symbol t of a stream uses table bits[...] - 1 of its position
  const uint8_t *bits;
  int32_t syms_per_pos, streams_per_session, n_tables;
  // reconstruction inside the decoder (rans_decode_chain_kernel with candidates)
  ReconView recon;
};

// Offset (in table entries of `stride` each) of the table that the 32 symbols from unit-relative group g on use.
__device__ __forceinline__ uint32_t group_table(const RansArgs &a, int64_t stream, int64_t begin, int32_t g,
                                                uint32_t stride, bool *bad) {
  // (a stream has fewer than 2^31 symbols and there are fewer than 2^31 streams: 32-bit divisions)
  const uint32_t spp = (uint32_t)a.syms_per_pos;
  const uint32_t pos = (uint32_t)(begin + (int64_t)g * kLanes) / spp;
  const uint32_t n_pos = (uint32_t)a.syms_per_stream / spp;
  int b = a.bits[(int64_t)((uint32_t)stream / (uint32_t)a.streams_per_session) * n_pos + pos];
  if (b < 1 || b > a.n_tables) {
    *bad = true;
    b = 1;
  }
  return (uint32_t)(b - 1) * stride;
}

// Frequencies of symbols 4*lane .. 4*lane+3 and the cumulative frequency in
// front of them, for all 64 lanes of a wavefront.  Returns the table's total.
__device__ __forceinline__ uint32_t load_freq4(const uint16_t *freq, int lane, uint32_t f[4], uint32_t *cum0) {
  const uint2 fv = *reinterpret_cast<const uint2 *>(freq + lane * 4);
  f[0] = fv.x & 0xffffu;
  f[1] = fv.x >> 16;
  f[2] = fv.y & 0xffffu;
  f[3] = fv.y >> 16;
  const uint32_t sum = f[0] + f[1] + f[2] + f[3];
  const uint32_t inc = wave_inclusive_scan(sum);
  *cum0 = inc - sum;
  return __shfl(inc, 63, 64);
}

__device__ __forceinline__ void wave_sync() {
  // LDS traffic of one wavefront executes in order; this only stops the
  // compiler from moving LDS accesses across a staging boundary.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// A workgroup barrier that orders LDS traffic only: what the wavefront wrote to LDS is there when the others
// pass, and its global loads and stores stay in flight (__syncthreads waits for those too, and a store to HBM
// takes the better part of a microsecond to be acknowledged).
__device__ __forceinline__ void lds_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0), vmcnt and expcnt left alone
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// ---------------------------------------------------------------------------
// Encoder
// ---------------------------------------------------------------------------
// Table entry per symbol (16 bytes).  A step is
//     if x > thr: emit (x & 0xffff), x >>= 16        thr = f * 2^20 - 1  (f = 4096: 2^32 - 1)
//     x' = q * (4096 - f) + x + cum                  q = floor(x / f)
// and differs only in how the exact quotient is formed:
//   short form, usable when every f of the table is <= 2048 (the normal case):
//       q = mulhi(x, m) >> s   with s = ceil(log2 f) - 1, m = ceil(2^(32+s) / f).
//     Exact because x < f * 2^20 after the renormalisation: the error term x * (m*f - 2^(32+s))
//     stays below 2^(32+s) as long as f^2 <= 2^(12+s), i.e. s <= 10.  For f = 1 the multiplier
//     2^32 - 1 yields x - 1, and the missing 4095 is added to the entry's cum.
//       .x = m   .y = thr   .z = (4096 - f) | s << 24   .w = cum (+4095 if f = 1)
//   long form, for tables with an f > 2048: a reciprocal of 33 bits, 2^32 + m = floor(2^(32+l) / f) + 1 with
//   l = ceil(log2 f), whose leading bit is implied:
//       q = (mulhi(m, x) + x) >> l
//     Exact because the error term x * ((2^32 + m) * f - 2^(32+l)) <= x * f < f^2 * 2^20 <= 2^(32+l) for
//     l <= 12; and x * (2^32 + m) stays below 2^64 (x / f < 2^20), so the sum does not overflow.
//       .x = m   .y = thr   .z = (4096 - f) | l << 24   .w = cum
// A symbol with f = 0 gets .w = 1 << 31, which is collected and reported if it occurs in the data.
template <bool LONG>
__device__ __forceinline__ uint4 make_enc_entry(uint32_t f, uint32_t cum) {
  if (f == 0) return make_uint4(0u, 0xffffffffu, 0u, 0x80000000u);
  const uint32_t l = f > 1 ? 32u - (uint32_t)__builtin_clz(f - 1) : 0u;  // ceil(log2 f)
  const uint32_t thr = f >= kScale ? 0xffffffffu : (f << 20) - 1u;
  if (LONG) {
    // floor((2^l - f) * 2^32 / f) by two 32-bit divisions (numerators stay below 2^28)
    const uint32_t n = (1u << l) - f;
    const uint32_t q1 = (n << 16) / f, r1 = (n << 16) - q1 * f;
    const uint32_t m = (q1 << 16) + (r1 << 16) / f + 1u;
    return make_uint4(m, thr, (kScale - f) | (l << 24), cum & 0xfffu);
  }
  if (f == 1) return make_uint4(0xffffffffu, thr, kScale - 1u, (cum & 0xfffu) + (kScale - 1u));
  // ceil(2^(32+s) / f), s = l - 1, as 2^32 * 2^s / f: again two divisions with small numerators
  const uint32_t s = l - 1u;
  const uint32_t n = 1u << s;  // n < f
  const uint32_t q1 = (n << 16) / f, r1 = (n << 16) - q1 * f;
  const uint32_t q2 = (r1 << 16) / f, r2 = (r1 << 16) - q2 * f;
  const uint32_t m = (q1 << 16) + q2 + (r2 ? 1u : 0u);
  return make_uint4(m, thr, (kScale - f) | (s << 24), cum & 0xfffu);
}

// One coding step.  Every lane stores its low 16 bits each time -- the emitting lanes into the word
// list, the others into a scratch slot of their own -- so that the step has no branch; `on` (MASKED
// only) is false for lanes that hold no symbol in a ragged group.
template <bool LONG, bool MASKED>
__device__ __forceinline__ void enc_step(uint32_t &x, const uint4 e, uint16_t *&wtop, uint16_t *scratch,
                                         uint32_t &flags, uint32_t below, bool on) {
  uint32_t m32 = (uint32_t)__builtin_amdgcn_uicmp(x, e.y, 34 /* unsigned > */);
  bool emit = x > e.y;
  if (MASKED) {
    emit = emit && on;
    m32 = (uint32_t)__builtin_amdgcn_ballot_w64(emit);
  }
  // hardware lane h carries rANS lane 31 - h, which the encoder visits first for h = 0; `below` is the
  // mask of the lanes under this one within its half, so that a mirror lane ranks like its twin
  // (`wtop` = next free slot of the batch's word list, uniform)
  uint16_t *slot = wtop + __builtin_popcount(m32 & below);
  *(emit ? slot : scratch) = (uint16_t)x;
  x = emit ? x >> 16 : x;
  wtop += __builtin_popcount(m32);
  uint32_t xn;
  if (LONG) {
    const uint32_t q = (__umulhi(e.x, x) + x) >> (e.z >> 24);
    xn = __umul24(q, e.z) + (x + e.w);
  } else {
    const uint32_t q = __umulhi(e.x, x) >> (e.z >> 24);
    xn = __umul24(q, e.z) + (x + e.w);
  }
  if (MASKED) {
    x = on ? xn : x;
    flags |= on ? e.w : 0u;
  } else {
    x = xn;
    flags |= e.w;
  }
}

// The same step for the unrolled batches, with its instruction order pinned.  A wavefront issues in
// order and a dependent VALU result takes about two issue slots to arrive (measured on gfx950: 8.5
// cycles dependent, 4.3 independent).  The step has two dependent chains that both start at the
// compare -- the state update and the address of the word to store -- so they are interleaved one for
// one; left to itself the compiler emits them one after the other and the wavefront idles.
#define PLC_PIN() __builtin_amdgcn_sched_barrier(0)

template <bool LONG>
__device__ __forceinline__ void enc_step_pinned(uint32_t &x, const uint4 e, uint16_t *&wtop, uint16_t *scratch,
                                                uint32_t &flags, uint32_t below) {
  const uint32_t m32 = (uint32_t)__builtin_amdgcn_uicmp(x, e.y, 34 /* unsigned > */);
  const bool emit = x > e.y;
  PLC_PIN();
  const uint32_t x16 = x >> 16;
  PLC_PIN();
  const uint32_t under = m32 & below;
  PLC_PIN();
  const uint32_t xr = emit ? x16 : x;
  PLC_PIN();
  const uint32_t rank = (uint32_t)__builtin_popcount(under);
  PLC_PIN();
  const uint32_t t1 = __umulhi(e.x, xr);
  PLC_PIN();
  uint16_t *slot = wtop + rank;
  PLC_PIN();
  uint32_t q, xc;
  if (LONG) {
    q = (t1 + xr) >> (e.z >> 24);
  } else {
    q = t1 >> (e.z >> 24);
  }
  xc = xr + e.w;
  PLC_PIN();
  slot = emit ? slot : scratch;
  PLC_PIN();
  const uint32_t p = __umul24(q, e.z);
  PLC_PIN();
  *slot = (uint16_t)x;
  PLC_PIN();
  wtop += __builtin_popcount(m32);
  PLC_PIN();
  x = p + xc;
  PLC_PIN();
  flags |= e.w;
}

template <int W, bool ADAPT>
__global__ __launch_bounds__(W * 64) void rans_encode_kernel(const RansArgs a) {
  __shared__ uint4 table[ADAPT ? PLC_MAX_BITS * 256 : 256];
  __shared__ uint16_t table_of_group[ADAPT ? W : 1][2][kSuperGroups];  // ADAPT: table offset of each staged group
  __shared__ __attribute__((aligned(16))) uint8_t sym_stage[W][2][kSymStage];
  __shared__ __attribute__((aligned(16))) uint16_t word_stage[W][kBatchSyms + 8 + 64];  // list + carry + scratch slots
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t stream = blockIdx.x / a.wgs_per_stream;
  const int64_t chunk = (int64_t)(blockIdx.x - stream * a.wgs_per_stream) * W + wave;
  const bool live = chunk < a.units_per_stream;

  bool long_form = false;
  if (!ADAPT) {  // every wavefront scans the frequencies; entry 4*lane + r is built by wavefront (4*lane + r) mod W
    uint32_t f[4], cum;
    const uint32_t total = load_freq4(a.freq + stream * 256, lane, f, &cum);
    if (total != kScale && threadIdx.x == 0) raise(a.status, PLC_ERR_INVALID);
    long_form = __ballot(f[0] > 2048u || f[1] > 2048u || f[2] > 2048u || f[3] > 2048u) != 0;  // uniform
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int s = lane * 4 + r;
      if ((s & (W - 1)) == wave)
        table[s] = long_form ? make_enc_entry<true>(f[r], cum) : make_enc_entry<false>(f[r], cum);
      cum += f[r];
    }
  } else {  // one table per bit depth; an all-zero table (a depth the stream does not use) holds only invalid entries
    uint32_t f[PLC_MAX_BITS][4], cum[PLC_MAX_BITS];
    for (int t = 0; t < a.n_tables; ++t) {
      const uint32_t total = load_freq4(a.freq + (stream * a.n_tables + t) * 256, lane, f[t], &cum[t]);
      if (total != kScale && total != 0 && threadIdx.x == 0) raise(a.status, PLC_ERR_INVALID);
      long_form = long_form || __ballot(f[t][0] > 2048u || f[t][1] > 2048u || f[t][2] > 2048u || f[t][3] > 2048u) != 0;
    }
    for (int t = 0; t < a.n_tables; ++t) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int s = lane * 4 + r;
        if ((s & (W - 1)) == wave)
          table[t * 256 + s] = long_form ? make_enc_entry<true>(f[t][r], cum[t]) : make_enc_entry<false>(f[t][r], cum[t]);
        cum[t] += f[t][r];
      }
    }
  }
  __syncthreads();
  if (!live) return;  // no workgroup barrier below

  const int64_t unit = stream * a.units_per_stream + chunk;
  const int64_t begin = chunk * a.unit_syms;
  const int64_t rest = a.syms_per_stream - begin;
  const uint32_t len = (uint32_t)(rest < a.unit_syms ? rest : a.unit_syms);
  const uint8_t *ubase = a.sym_in + stream * a.syms_per_stream + begin;
  const uint32_t mis = (uint32_t)(reinterpret_cast<uintptr_t>(ubase) & 15u);
  const int32_t G = (int32_t)((len + kLanes - 1) / kLanes);
  const uint32_t top_syms = len - (uint32_t)(G - 1) * kLanes;  // symbols in the last group, 1..32
  uint16_t *wp = a.words_out + a.word_off[unit];
  uint16_t *wstage = word_stage[wave];
  uint16_t *scratch = wstage + kBatchSyms + 8 + lane;

  const int rl = 31 - (lane & 31);  // rANS lane carried by this hardware lane
  const uint32_t below = (1u << (lane & 31)) - 1u;
  const bool coder = lane < kLanes;
  const bool top_active = (uint32_t)rl < top_syms;
  uint32_t x = kLow, flags = 0;

  // Staging rounds walk the groups from the top, 64 groups per round (the first round takes what is
  // left over).  A round's symbols [32*glo, 32*ghi) are fetched as 16-byte pieces aligned in absolute
  // address and placed so that symbol (group ghi-1-j, lane l) always sits at  mis + l + 32 * (63 - j).
  bool bad_depth = false;
  // ADAPT: the table of the group that stage position `lane` will hold (group ghi - 64 + lane), fetched with the symbols
  auto group_load = [&](int32_t glo, int32_t ghi) -> uint32_t {
    const int32_t g = ghi - kSuperGroups + lane;
    if (!ADAPT || ghi <= 0 || g < (glo > 0 ? glo : 0) || g >= ghi) return 0u;
    return group_table(a, stream, begin, g, 256u, &bad_depth);
  };
  auto stage_load = [&](int32_t glo, int32_t ghi, uint4 v[kStagePieces], bool take[kStagePieces]) {
    // byte offsets relative to the unit's first symbol; pointers are formed by plain pointer arithmetic
    // on the kernel argument so that the loads stay global (not flat) memory instructions
    const int64_t lo = (int64_t)(glo > 0 ? glo : 0) * kLanes;
    int64_t hi = (int64_t)(ghi > 0 ? ghi : 0) * kLanes;
    hi = hi < (int64_t)len ? hi : (int64_t)len;
#pragma unroll
    for (int i = 0; i < kStagePieces; ++i) {
      const int64_t off = lo - (int64_t)mis + (int64_t)(lane + 64 * i) * 16;  // 16-byte aligned in absolute address
      take[i] = ghi > 0 && off < hi;
      if (take[i]) v[i] = load16_stream(ubase + off);
    }
  };
  auto stage_store = [&](int buf, int32_t cnt, const uint4 v[kStagePieces], const bool take[kStagePieces]) {
#pragma unroll
    for (int i = 0; i < kStagePieces; ++i)
      if (take[i])
        *reinterpret_cast<uint4 *>(&sym_stage[wave][buf][(lane + 64 * i) * 16 + kLanes * (kSuperGroups - cnt)]) = v[i];
  };
  // Words leave through an LDS list whose position p stands for the word at 16-byte-aligned address
  // (wp - pad) + vbase + p: the first `pad` positions of the unit are padding in front of its first word.
  // After each batch the complete 16-byte pieces are stored, one per lane, and the incomplete tail (< 8
  // words) moves to the front of the list.  Pieces that touch the padding or the end of the unit's
  // reservation are stored word by word.
  // (All of this bookkeeping is uniform; readfirstlane keeps it in scalar registers.)
  const uint32_t pad = __builtin_amdgcn_readfirstlane((uint32_t)((reinterpret_cast<uintptr_t>(wp) >> 1) & 7u));
  const uint32_t cap = a.word_cap < 0x7fffffffull ? (uint32_t)a.word_cap : 0x7fffffffu;  // a unit has < 2^31 symbols
  uint32_t vbase = 0;   // multiple of 8
  uint32_t fill = pad;  // positions of the list in use
  auto store_words = [&](uint32_t first_pos, uint32_t n_pos) {  // word-by-word, with all checks
    for (uint32_t p = first_pos + lane; p < first_pos + n_pos; p += 64) {
      const uint32_t v = vbase + p;
      if (v >= pad && v - pad < cap) wp[v - pad] = wstage[p];
    }
  };
  auto drain = [&](uint32_t new_fill_v) {
    const uint32_t new_fill = __builtin_amdgcn_readfirstlane(new_fill_v);
    wave_sync();
    const uint32_t full = new_fill / 8;  // at most 65 pieces
    const bool plain = vbase >= pad && vbase + 8 * full - pad <= cap;
    if (plain) {
      uint16_t *dst = wp + (vbase - pad);  // 16-byte aligned
      if ((uint32_t)lane < full)
        *reinterpret_cast<uint4 *>(dst + 8 * lane) = *reinterpret_cast<const uint4 *>(wstage + 8 * lane);
      if (full > 64 && lane == 0)
        *reinterpret_cast<uint4 *>(dst + 8 * 64) = *reinterpret_cast<const uint4 *>(wstage + 8 * 64);
    } else {
      store_words(0, 8 * full);
    }
    const uint32_t rest = new_fill - 8 * full;
    uint16_t carry = 0;
    if ((uint32_t)lane < rest) carry = wstage[8 * full + lane];
    wave_sync();
    if ((uint32_t)lane < rest) wstage[lane] = carry;
    vbase += 8 * full;
    fill = rest;
    wave_sync();
  };

  int32_t ghi = G;
  int32_t cnt_groups = G % kSuperGroups ? G % kSuperGroups : kSuperGroups;
  // groups of the first round that do not fill a batch (and the top group if it is ragged) run in a
  // rolled loop with lane masking; every other batch is 16 full groups, fully unrolled
  int32_t head_groups = cnt_groups % kBatch;
  if (head_groups == 0 && top_syms < kLanes) head_groups = kBatch;
  {
    uint4 v[kStagePieces];
    bool take[kStagePieces];
    stage_load(ghi - cnt_groups, ghi, v, take);
    stage_store(0, cnt_groups, v, take);
    if (ADAPT) table_of_group[wave][0][lane] = (uint16_t)group_load(ghi - cnt_groups, ghi);
  }
  wave_sync();
  int buf = 0;
  while (ghi > 0) {
    const int32_t glo = ghi - cnt_groups;
    uint4 nv[kStagePieces];
    bool ntake[kStagePieces];
    stage_load(glo - kSuperGroups, glo, nv, ntake);  // next round, in flight while this one is coded
    const uint32_t ngt = group_load(glo - kSuperGroups, glo);
    const uint16_t *gt = table_of_group[ADAPT ? wave : 0][buf];  // group j from the round's top sits at 63 - j
    const uint8_t *sb = &sym_stage[wave][buf][mis + rl];
    int32_t j0 = 0;
    // The prefetched round is written to LDS after the first batch of this round and BEFORE that batch's
    // words are stored: waiting for the loads then does not also wait for freshly issued stores (loads
    // and stores share one counter).
    bool landed = false;
    if (head_groups) {
      uint16_t *wtop = wstage + fill;
      for (int32_t j = 0; j < head_groups; ++j) {
        const uint4 e = table[sb[kLanes * (kSuperGroups - 1 - j)] + (ADAPT ? gt[kSuperGroups - 1 - j] : 0u)];
        if (long_form) {
          enc_step<true, true>(x, e, wtop, scratch, flags, below, j != 0 || top_active);
        } else {
          enc_step<false, true>(x, e, wtop, scratch, flags, below, j != 0 || top_active);
        }
      }
      stage_store(buf ^ 1, kSuperGroups, nv, ntake);
      if (ADAPT) table_of_group[wave][buf ^ 1][lane] = (uint16_t)ngt;
      landed = true;
      drain((uint32_t)(wtop - wstage));
      j0 = head_groups;
    }
    for (; j0 < cnt_groups; j0 += kBatch) {
      const uint8_t *sbb = sb + kLanes * (kSuperGroups - kBatch - j0);  // lowest group of this batch
      uint32_t sy[kBatch];
      uint16_t *wtop = wstage + fill;
#pragma unroll
      for (int j = 0; j < kBatch; ++j) sy[j] = sbb[kLanes * (kBatch - 1 - j)];
      if (ADAPT) {
        const uint16_t *gtb = gt + (kSuperGroups - kBatch - j0);
#pragma unroll
        for (int j = 0; j < kBatch; ++j) sy[j] += gtb[kBatch - 1 - j];
      }
      // table entries are fetched four groups ahead of the chain, so that their LDS time hides behind it
      uint4 e[2][4];
#pragma unroll
      for (int j = 0; j < 4; ++j) e[0][j] = table[sy[j]];
#pragma unroll
      for (int qt = 0; qt < kBatch / 4; ++qt) {
        if (qt + 1 < kBatch / 4) {
#pragma unroll
          for (int j = 0; j < 4; ++j) e[(qt + 1) & 1][j] = table[sy[4 * (qt + 1) + j]];
        }
        if (long_form) {
#pragma unroll
          for (int j = 0; j < 4; ++j) enc_step_pinned<true>(x, e[qt & 1][j], wtop, scratch, flags, below);
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j) enc_step_pinned<false>(x, e[qt & 1][j], wtop, scratch, flags, below);
        }
      }
      if (!landed) {
        stage_store(buf ^ 1, kSuperGroups, nv, ntake);
        if (ADAPT) table_of_group[wave][buf ^ 1][lane] = (uint16_t)ngt;
        landed = true;
      }
      drain((uint32_t)(wtop - wstage));
    }
    wave_sync();
    buf ^= 1;
    ghi = glo;
    cnt_groups = kSuperGroups;
    head_groups = 0;
  }
  if (coder) a.states_out[unit * kLanes + rl] = x;
  store_words(0, fill);  // the incomplete last piece
  const uint32_t n_words = vbase + fill - pad;
  if (lane == 0) {
    a.n_words_out[unit] = n_words;
    if ((uint64_t)n_words > a.word_cap) raise(a.status, PLC_ERR_CAPACITY);
  }
  if (coder && (flags & 0x80000000u)) raise(a.status, PLC_ERR_INVALID);  // a symbol with f = 0 occurred
  if (bad_depth) raise(a.status, PLC_ERR_INVALID);
}

// ---------------------------------------------------------------------------
// Encoder for many units: two units per wavefront
// ---------------------------------------------------------------------------
// With thousands of units in flight the kernel above is bound by instruction issue, not by latency (measured:
// 83 cycles of a SIMD per step of a unit, the ~21 instructions of a step at 4 cycles each), and half of every
// instruction's lanes only mirror the other half.  Here lanes 32-63 code a unit of their own: the step's
// instructions are the same, only the word positions are per half -- a lane ranks itself inside its own
// half of the compare's lane mask, and the list pointer is a per-lane value that advances by its half's
// count.  The two units of a wavefront have the same length: two consecutive whole chunks of a stream (one
// table), or two consecutive whole streams (TWO_TABLES); a unit without such a partner (an odd count, a
// shorter last chunk) is coded by the lower half while the upper half shadows it and stores nothing.
// Symbols and words are staged per half exactly as above.
template <bool LONG, bool MASKED>
__device__ __forceinline__ void enc2_step(uint32_t &x, const uint4 e, uint16_t *&wtop, uint16_t *scratch,
                                          uint32_t &flags, uint32_t below, bool upper, bool on) {
  bool emit = x > e.y;
  if (MASKED) emit = emit && on;
  const uint64_t m = __builtin_amdgcn_ballot_w64(emit);
  const uint32_t mine = upper ? (uint32_t)(m >> 32) : (uint32_t)m;  // the emit mask of this lane's half
  uint16_t *slot = wtop + __builtin_popcount(mine & below);
  *(emit ? slot : scratch) = (uint16_t)x;
  x = emit ? x >> 16 : x;
  wtop += __builtin_popcount(mine);
  const uint32_t t1 = __umulhi(e.x, x);
  const uint32_t q = (LONG ? t1 + x : t1) >> (e.z >> 24);
  const uint32_t xn = __umul24(q, e.z) + (x + e.w);
  if (MASKED) {
    x = on ? xn : x;
    flags |= on ? e.w : 0u;
  } else {
    x = xn;
    flags |= e.w;
  }
}

template <bool LONG>
__device__ __forceinline__ void enc2_step_pinned(uint32_t &x, const uint4 e, uint16_t *&wtop, uint16_t *scratch,
                                                 uint32_t &flags, uint32_t below, bool upper) {
  const uint64_t m = __builtin_amdgcn_uicmp(x, e.y, 34 /* unsigned > */);
  const bool emit = x > e.y;
  PLC_PIN();
  const uint32_t x16 = x >> 16;
  PLC_PIN();
  const uint32_t mine = upper ? (uint32_t)(m >> 32) : (uint32_t)m;
  PLC_PIN();
  const uint32_t xr = emit ? x16 : x;
  PLC_PIN();
  const uint32_t under = mine & below;
  PLC_PIN();
  const uint32_t t1 = __umulhi(e.x, xr);
  PLC_PIN();
  const uint32_t rank = (uint32_t)__builtin_popcount(under);
  PLC_PIN();
  uint32_t q, xc;
  if (LONG) {
    q = (t1 + xr) >> (e.z >> 24);
  } else {
    q = t1 >> (e.z >> 24);
  }
  xc = xr + e.w;
  PLC_PIN();
  uint16_t *slot = wtop + rank;
  PLC_PIN();
  const uint32_t p = __umul24(q, e.z);
  PLC_PIN();
  slot = emit ? slot : scratch;
  PLC_PIN();
  wtop += __builtin_popcount(mine);
  PLC_PIN();
  *slot = (uint16_t)x;
  PLC_PIN();
  x = p + xc;
  PLC_PIN();
  flags |= e.w;
}

constexpr int kPairMaxWaves = 4;
// SUPER = batches of symbols staged per round.  Four, as above, is the efficient size (a round's bookkeeping is
// spread over 64 steps).  With whole streams a workgroup is one wavefront with two tables, and its LDS decides
// how many are resident: 18.8 KB with four batches (eight per compute unit), 14.7 KB with two (eleven).  Two is
// taken only where it lets every pair of streams be resident at once instead of leaving a second, mostly empty
// round (5120 streams: 3.3 -> 2.5 ms); where there are several full rounds anyway the shorter rounds cost more
// than the extra wavefronts gain (16,384 streams: 7.4 against 7.7 ms).
template <int W, bool TWO_TABLES, int SUPER = 4>
__global__ __launch_bounds__(W * 64) void rans_encode_pair_kernel(const RansArgs a) {
  constexpr int kPairGroups = SUPER * kBatch;                  // groups per staging round
  constexpr int kPairSymStage = kPairGroups * kLanes + 32;     // its symbols at any 16-byte misalignment
  constexpr int kPairPieces = (kPairSymStage + 1023) / 1024;   // 16-byte pieces per lane and round
  static_assert(!TWO_TABLES || W == 1, "whole streams: one pair of streams per workgroup");
  __shared__ uint4 table[TWO_TABLES ? 2 : 1][256];
  __shared__ __attribute__((aligned(16))) uint8_t sym_stage[W][2][2][kPairSymStage];                // [half][buffer]
  __shared__ __attribute__((aligned(16))) uint16_t word_stage[W][2][kBatchSyms + 8 + 64];       // list + carry + scratch slots
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int half = lane >> 5;
  const bool upper = half != 0;

  // ---- which units: unit[0] for lanes 0-31, unit[1] for lanes 32-63 (or none: the upper half then shadows unit[0])
  int64_t stream[2], begin[2];
  bool second;       // uniform: the upper half has a unit of its own
  bool live = true;  // uniform: this wavefront has a unit at all
  uint32_t len;
  if (TWO_TABLES) {
    stream[0] = 2 * (int64_t)blockIdx.x;
    second = stream[0] + 1 < a.n_units;
    stream[1] = second ? stream[0] + 1 : stream[0];
    begin[0] = begin[1] = 0;
    len = (uint32_t)a.syms_per_stream;
  } else {
    const int64_t st = blockIdx.x / a.pair_wgs_per_stream;
    const int64_t slot = (int64_t)(blockIdx.x - st * a.pair_wgs_per_stream) * W + wave;
    const int64_t n_full = a.syms_per_stream / a.unit_syms;  // chunks of full length
    const int64_t n_pairs = n_full / 2;
    int64_t chunk0;
    if (slot < n_pairs) {
      chunk0 = 2 * slot, second = true;
    } else if ((n_full & 1) && slot == n_pairs) {
      chunk0 = n_full - 1, second = false;                   // the odd full chunk
    } else {
      chunk0 = n_full, second = false;                       // the shorter last chunk
      live = slot == n_pairs + (n_full & 1) && n_full < a.units_per_stream;
    }
    stream[0] = stream[1] = st;
    begin[0] = chunk0 * a.unit_syms;
    begin[1] = second ? begin[0] + a.unit_syms : begin[0];
    const int64_t rest = a.syms_per_stream - begin[0];
    len = (uint32_t)(rest < a.unit_syms ? rest : a.unit_syms);
  }

  bool long_form = false;
  {  // table entries: every wavefront scans the frequencies; entry 4*lane + r is built by wavefront (4*lane + r) mod W
    uint32_t f[TWO_TABLES ? 2 : 1][4], cum[TWO_TABLES ? 2 : 1];
#pragma unroll
    for (int t = 0; t < (TWO_TABLES ? 2 : 1); ++t) {
      const uint32_t total = load_freq4(a.freq + stream[t] * 256, lane, f[t], &cum[t]);
      if (total != kScale && threadIdx.x == 0) raise(a.status, PLC_ERR_INVALID);
      long_form = long_form || __ballot(f[t][0] > 2048u || f[t][1] > 2048u || f[t][2] > 2048u || f[t][3] > 2048u) != 0;
    }
#pragma unroll
    for (int t = 0; t < (TWO_TABLES ? 2 : 1); ++t) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int s = lane * 4 + r;
        if ((s & (W - 1)) == wave)
          table[t][s] = long_form ? make_enc_entry<true>(f[t][r], cum[t]) : make_enc_entry<false>(f[t][r], cum[t]);
        cum[t] += f[t][r];
      }
    }
  }
  __syncthreads();
  if (!live) return;  // no workgroup barrier below

  const int64_t unit[2] = {stream[0] * a.units_per_stream + begin[0] / a.unit_syms,
                           stream[1] * a.units_per_stream + begin[1] / a.unit_syms};
  const uint8_t *ubase[2] = {a.sym_in + stream[0] * a.syms_per_stream + begin[0],
                             a.sym_in + stream[1] * a.syms_per_stream + begin[1]};
  const uint32_t mis[2] = {(uint32_t)(reinterpret_cast<uintptr_t>(ubase[0]) & 15u),
                           (uint32_t)(reinterpret_cast<uintptr_t>(ubase[1]) & 15u)};
  const int32_t G = (int32_t)((len + kLanes - 1) / kLanes);
  const uint32_t top_syms = len - (uint32_t)(G - 1) * kLanes;  // symbols in the last group, 1..32
  uint16_t *wp[2] = {a.words_out + a.word_off[unit[0]], a.words_out + a.word_off[unit[1]]};
  uint16_t *wstage = word_stage[wave][half];               // this lane's half's list
  uint16_t *scratch = wstage + kBatchSyms + 8 + (lane & 31);
  // (a shadowing upper half writes its words to its own LDS list and never to global memory)

  const int rl = 31 - (lane & 31);  // rANS lane carried by this hardware lane
  const uint32_t below = (1u << (lane & 31)) - 1u;
  const bool top_active = (uint32_t)rl < top_syms;
  const uint4 *mytable = table[TWO_TABLES ? half : 0];
  uint32_t x = kLow, flags = 0;

  // Symbol staging per half, as in the kernel above: a round's symbols are fetched as 16-byte pieces aligned
  // in absolute address by all 64 lanes and placed so that symbol (group ghi-1-j, lane l) sits at
  // mis + l + 32 * (kPairGroups - 1 - j).
  auto stage_load = [&](int h, int32_t glo, int32_t ghi, uint4 v[kPairPieces], bool take[kPairPieces]) {
    const int64_t lo = (int64_t)(glo > 0 ? glo : 0) * kLanes;
    int64_t hi = (int64_t)(ghi > 0 ? ghi : 0) * kLanes;
    hi = hi < (int64_t)len ? hi : (int64_t)len;
#pragma unroll
    for (int i = 0; i < kPairPieces; ++i) {
      const int64_t off = lo - (int64_t)mis[h] + (int64_t)(lane + 64 * i) * 16;  // 16-byte aligned in absolute address
      take[i] = ghi > 0 && off < hi;
      if (take[i]) v[i] = load16_stream(ubase[h] + off);
    }
  };
  auto stage_store = [&](int h, int buf, int32_t cnt, const uint4 v[kPairPieces], const bool take[kPairPieces]) {
#pragma unroll
    for (int i = 0; i < kPairPieces; ++i)
      if (take[i])
        *reinterpret_cast<uint4 *>(&sym_stage[wave][h][buf][(lane + 64 * i) * 16 + kLanes * (kPairGroups - cnt)]) = v[i];
  };
  // Word lists per half, as above: position p of a list stands for the word at 16-byte-aligned address
  // (wp - pad) + vbase + p.
  const uint32_t pad[2] = {(uint32_t)__builtin_amdgcn_readfirstlane((int)((reinterpret_cast<uintptr_t>(wp[0]) >> 1) & 7u)),
                           (uint32_t)__builtin_amdgcn_readfirstlane((int)((reinterpret_cast<uintptr_t>(wp[1]) >> 1) & 7u))};
  const uint32_t cap = a.word_cap < 0x7fffffffull ? (uint32_t)a.word_cap : 0x7fffffffu;  // a unit has < 2^31 symbols
  uint32_t vbase[2] = {0u, 0u};          // multiples of 8
  uint32_t fill[2] = {pad[0], pad[1]};   // positions of each list in use
  const bool writes[2] = {true, second};
  auto store_words = [&](int h, uint32_t first_pos, uint32_t n_pos) {  // word-by-word, with all checks
    if (!writes[h]) return;
    const uint16_t *list = word_stage[wave][h];
    for (uint32_t p = first_pos + lane; p < first_pos + n_pos; p += 64) {
      const uint32_t v = vbase[h] + p;
      if (v >= pad[h] && v - pad[h] < cap) wp[h][v - pad[h]] = list[p];
    }
  };
  auto drain = [&](int h, uint32_t new_fill) {  // new_fill uniform
    uint16_t *list = word_stage[wave][h];
    const uint32_t full = new_fill / 8;  // at most 65 pieces
    const bool plain = vbase[h] >= pad[h] && vbase[h] + 8 * full - pad[h] <= cap;
    if (plain) {
      if (writes[h]) {
        uint16_t *dst = wp[h] + (vbase[h] - pad[h]);  // 16-byte aligned
        if ((uint32_t)lane < full)
          *reinterpret_cast<uint4 *>(dst + 8 * lane) = *reinterpret_cast<const uint4 *>(list + 8 * lane);
        if (full > 64 && lane == 0)
          *reinterpret_cast<uint4 *>(dst + 8 * 64) = *reinterpret_cast<const uint4 *>(list + 8 * 64);
      }
    } else {
      store_words(h, 0, 8 * full);
    }
    const uint32_t rest = new_fill - 8 * full;
    uint16_t carry = 0;
    if ((uint32_t)lane < rest) carry = list[8 * full + lane];
    wave_sync();
    if ((uint32_t)lane < rest) list[lane] = carry;
    vbase[h] += 8 * full;
    fill[h] = rest;
  };
  // after a batch: each half's new fill from its lanes' list pointer (uniform inside a half), both lists drained
  auto drain_both = [&](uint16_t *wtop) {
    const uint32_t mine = (uint32_t)(wtop - wstage);
    const uint32_t f0 = (uint32_t)__builtin_amdgcn_readlane((int)mine, 0);
    const uint32_t f1 = (uint32_t)__builtin_amdgcn_readlane((int)mine, 32);
    wave_sync();
    drain(0, f0);
    drain(1, f1);
    wave_sync();
  };

  int32_t ghi = G;
  int32_t cnt_groups = G % kPairGroups ? G % kPairGroups : kPairGroups;
  // groups of the first round that do not fill a batch (and the top group if it is ragged) run in a
  // rolled loop with lane masking; every other batch is 16 full groups, fully unrolled
  int32_t head_groups = cnt_groups % kBatch;
  if (head_groups == 0 && top_syms < kLanes) head_groups = kBatch;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    uint4 v[kPairPieces];
    bool take[kPairPieces];
    stage_load(h, ghi - cnt_groups, ghi, v, take);
    stage_store(h, 0, cnt_groups, v, take);
  }
  wave_sync();
  int buf = 0;
  while (ghi > 0) {
    const int32_t glo = ghi - cnt_groups;
    uint4 nv[2][kPairPieces];
    bool ntake[2][kPairPieces];
#pragma unroll
    for (int h = 0; h < 2; ++h) stage_load(h, glo - kPairGroups, glo, nv[h], ntake[h]);  // next round, in flight
    const uint8_t *sb = &sym_stage[wave][half][buf][(upper ? mis[1] : mis[0]) + rl];
    int32_t j0 = 0;
    bool landed = false;
    if (head_groups) {
      uint16_t *wtop = wstage + (upper ? fill[1] : fill[0]);
      for (int32_t j = 0; j < head_groups; ++j) {
        const uint4 e = mytable[sb[kLanes * (kPairGroups - 1 - j)]];
        if (long_form) {
          enc2_step<true, true>(x, e, wtop, scratch, flags, below, upper, j != 0 || top_active);
        } else {
          enc2_step<false, true>(x, e, wtop, scratch, flags, below, upper, j != 0 || top_active);
        }
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) stage_store(h, buf ^ 1, kPairGroups, nv[h], ntake[h]);
      landed = true;
      drain_both(wtop);
      j0 = head_groups;
    }
    for (; j0 < cnt_groups; j0 += kBatch) {
      const uint8_t *sbb = sb + kLanes * (kPairGroups - kBatch - j0);  // lowest group of this batch
      uint32_t sy[kBatch];
      uint16_t *wtop = wstage + (upper ? fill[1] : fill[0]);
#pragma unroll
      for (int j = 0; j < kBatch; ++j) sy[j] = sbb[kLanes * (kBatch - 1 - j)];
      // table entries are fetched four groups ahead of the chain, so that their LDS time hides behind it
      uint4 e[2][4];
#pragma unroll
      for (int j = 0; j < 4; ++j) e[0][j] = mytable[sy[j]];
#pragma unroll
      for (int qt = 0; qt < kBatch / 4; ++qt) {
        if (qt + 1 < kBatch / 4) {
#pragma unroll
          for (int j = 0; j < 4; ++j) e[(qt + 1) & 1][j] = mytable[sy[4 * (qt + 1) + j]];
        }
        if (long_form) {
#pragma unroll
          for (int j = 0; j < 4; ++j) enc2_step_pinned<true>(x, e[qt & 1][j], wtop, scratch, flags, below, upper);
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j) enc2_step_pinned<false>(x, e[qt & 1][j], wtop, scratch, flags, below, upper);
        }
      }
      if (!landed) {
#pragma unroll
        for (int h = 0; h < 2; ++h) stage_store(h, buf ^ 1, kPairGroups, nv[h], ntake[h]);
        landed = true;
      }
      drain_both(wtop);
    }
    wave_sync();
    buf ^= 1;
    ghi = glo;
    cnt_groups = kPairGroups;
    head_groups = 0;
  }
  if (!upper || second) a.states_out[(upper ? unit[1] : unit[0]) * kLanes + rl] = x;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    store_words(h, 0, fill[h]);  // the incomplete last piece
    const uint32_t n_words = vbase[h] + fill[h] - pad[h];
    if (lane == 0 && writes[h]) {
      a.n_words_out[unit[h]] = n_words;
      if ((uint64_t)n_words > a.word_cap) raise(a.status, PLC_ERR_CAPACITY);
    }
  }
  if ((!upper || second) && (flags & 0x80000000u)) raise(a.status, PLC_ERR_INVALID);  // a symbol with f = 0 occurred
}

// ---------------------------------------------------------------------------
// Encoder for few, long units: three wavefronts per unit
// ---------------------------------------------------------------------------
// When there are no more units than compute units, time is the length of one unit's chain of steps,
// and a lone wavefront issues in order: an independent vector instruction every ~4.3 cycles, one that needs
// the previous result after ~9, an LDS instruction every 8-16.  So everything that is not the state
// recurrence moves to two helper wavefronts of the same workgroup, which run on other SIMDs of the compute
// unit:
//   feeder  stages the symbols (64 groups ahead, as above) and turns every (group, lane) of the next
//           batch into its 16-byte table entry at a fixed place of an LDS ring; a lane without a symbol
//           (ragged top group, or a step past the unit's first group) gets an identity entry;
//   coder   per step: one LDS read of its entry, one LDS write of its state before the step, and the
//           recurrence itself -- no ranking, no addresses to compute, no branches;
//   packer  one batch behind, recovers from the stored states which lanes emitted (x > thr), ranks
//           them with one ballot per two steps, packs the 16-bit words and writes them out.
// The three meet at one workgroup barrier per batch of 16 steps.
constexpr int kEntrySlots = 3;  // feeder writes b+1, coder reads b, packer reads b-1
constexpr int kStateSlots = 2;  // coder writes b, packer reads b-1
constexpr int kIdentity = PLC_MAX_BITS * 256;  // table index of the entry that leaves a state unchanged
// These kernels hold two units per compute unit (LDS), 512 at a time, and a unit's time is that of its chain:
// up to two rounds they beat the many-unit kernels (768 units: encode 1.7 against 2.8 ms, decode 3.3 against
// 4.9 ms), at three they tie with them.
constexpr int64_t kPipeMaxUnits = 1024;
constexpr int64_t kChainMaxUnits = 1024;  // the same bound for the decoder of whole-stream units
// The decoder with one table per depth holds one unit per compute unit (its tables take 128 KB of LDS): two
// rounds of 256 are what it may take before the many-unit decoder is as fast.
constexpr int64_t kDepthsMaxUnits = 512;
// From this many streams on (more than two workgroups per compute unit) the decoder that reconstructs takes
// its three-block ring where k <= 4 lets three workgroups share a compute unit.
constexpr int64_t kComputeUnits = 256;  // MI355X
constexpr int64_t kDenseStreams = 512;
constexpr int kCompactMaxK = 4;  // up to here four workgroups of the decoder with 4-byte entries fit a compute unit
constexpr int kDenseMaxK = 6;  // up to here the kernel's registers (156 at k = 6) leave room for three wavefronts per SIMD

template <bool LONG>
__device__ __forceinline__ void pipe_step(uint32_t &x, const uint4 e) {
  const bool emit = x > e.y;
  const uint32_t xr = emit ? x >> 16 : x;
  const uint32_t t1 = __umulhi(e.x, xr);
  const uint32_t q = (LONG ? t1 + xr : t1) >> (e.z >> 24);
  x = __umul24(q, e.z) + (xr + e.w);
}

// One batch of the coder.  Entries are fetched kAhead steps before their use, so that the LDS round
// trip (longer than a step while the helpers are busy on the same LDS) stays off the chain.
template <bool LONG>
__device__ __forceinline__ void pipe_batch(uint32_t &x, const uint4 *eb, uint32_t *xb) {
  constexpr int kAhead = 4;
  uint4 e[kAhead];
#pragma unroll
  for (int j = 0; j < kAhead; ++j) e[j] = eb[j * kLanes];
  uint32_t x_even = 0;
#pragma unroll
  for (int j = 0; j < kBatch; ++j) {
    const uint4 cur = e[j % kAhead];
    PLC_PIN();
    if (j + kAhead < kBatch) e[j % kAhead] = eb[(j + kAhead) * kLanes];
    if (j & 1) {  // the states before steps j - 1 and j leave in one LDS instruction
      xb[(j - 1) * kLanes] = x_even;
      xb[j * kLanes] = x;
    } else {
      x_even = x;
    }
    PLC_PIN();
    pipe_step<LONG>(x, cur);
  }
}

template <bool ADAPT>  // ADAPT: one table per bit depth (the *_bucketed call)
__global__ __launch_bounds__(192) void rans_encode_pipe_kernel(const RansArgs a) {
  __shared__ uint4 table[kIdentity + 1];
  __shared__ uint16_t table_of_group[2][kSuperGroups];  // ADAPT: table offset of each group of a staging round
  __shared__ uint4 entry_ring[kEntrySlots][kBatch][kLanes];
  __shared__ uint32_t state_ring[kStateSlots][kBatch][kLanes];
  __shared__ __attribute__((aligned(16))) uint8_t sym_stage[2][kSymStage];
  __shared__ __attribute__((aligned(16))) uint16_t word_stage[2 * kBatchSyms + 8 + 64];  // list, carry, idle slots
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t unit = blockIdx.x;  // one unit per stream, one workgroup per unit

  bool long_form = false;
  {  // every wavefront scans the frequencies; of a lane's four entries the coder builds one, the feeder
     // one and the packer two
    const int n_tables = ADAPT ? a.n_tables : 1;
    uint32_t f[ADAPT ? PLC_MAX_BITS : 1][4], cum[ADAPT ? PLC_MAX_BITS : 1];
    for (int t = 0; t < n_tables; ++t) {
      const uint32_t total = load_freq4(a.freq + (unit * n_tables + t) * 256, lane, f[t], &cum[t]);
      if (total != kScale && !(ADAPT && total == 0) && threadIdx.x == 0) raise(a.status, PLC_ERR_INVALID);
      long_form = long_form || __ballot(f[t][0] > 2048u || f[t][1] > 2048u || f[t][2] > 2048u || f[t][3] > 2048u) != 0;
    }
    for (int t = 0; t < n_tables; ++t) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if ((r < 2 ? r : 2) == wave)
          table[t * 256 + lane * 4 + r] =
              long_form ? make_enc_entry<true>(f[t][r], cum[t]) : make_enc_entry<false>(f[t][r], cum[t]);
        cum[t] += f[t][r];
      }
    }
    if (threadIdx.x == 0) table[kIdentity] = make_uint4(0u, 0xffffffffu, 0u, 0u);  // never emits, x' = x
  }
  __syncthreads();

  const uint32_t len = (uint32_t)a.syms_per_stream;
  const uint8_t *ubase = a.sym_in + unit * a.syms_per_stream;
  const uint32_t mis = (uint32_t)(reinterpret_cast<uintptr_t>(ubase) & 15u);
  const int32_t G = (int32_t)((len + kLanes - 1) / kLanes);
  // Batch 0 holds the top G mod 16 groups (a full 16 if that is 0) followed by identity steps; every
  // later batch is 16 full groups.  Batch b codes groups top(b)-1 down to top(b)-16.
  const int32_t head = G % kBatch ? G % kBatch : kBatch;
  const int32_t n_batches = (G - head) / kBatch + 1;
  auto batch_top = [&](int32_t b) { return b == 0 ? G : G - head - (b - 1) * kBatch; };
  // Symbol staging rounds of four batches; a round's buffer starts at the 16-byte-aligned address at or
  // below its lowest symbol, so the symbol at unit offset t sits at  t - 32 * bottom + mis.
  auto round_bottom = [&](int32_t r) {
    const int32_t g = batch_top(4 * r + 3) - kBatch;
    return g > 0 ? g : 0;
  };
  const int32_t n_rounds = (n_batches + 3) / 4;

  uint32_t x = kLow;              // coder
  bool bad_symbol = false;        // feeder
  bool bad_depth = false;
  uint4 nv[kStagePieces];         // feeder: next round's symbols in flight
  bool ntake[kStagePieces];
  uint32_t ntog = 0;              // feeder, ADAPT: table offset of group bottom + lane of the next round
  // packer: the word list, as in the single-wavefront encoder
  uint16_t *wp = a.words_out + a.word_off[unit];
  const uint32_t pad = __builtin_amdgcn_readfirstlane((uint32_t)((reinterpret_cast<uintptr_t>(wp) >> 1) & 7u));
  const uint32_t cap = a.word_cap < 0x7fffffffull ? (uint32_t)a.word_cap : 0x7fffffffu;
  uint32_t vbase = 0, fill = pad;

  auto round_load = [&](int32_t r) {
    const int64_t lo = (int64_t)round_bottom(r) * kLanes;
    int64_t hi = (int64_t)batch_top(4 * r) * kLanes;
    hi = hi < (int64_t)len ? hi : (int64_t)len;
#pragma unroll
    for (int i = 0; i < kStagePieces; ++i) {
      const int64_t off = lo - (int64_t)mis + (int64_t)(lane + 64 * i) * 16;  // 16-byte aligned in absolute address
      ntake[i] = r < n_rounds && off < hi;
      if (ntake[i]) nv[i] = load16_stream(ubase + off);
    }
    if (ADAPT) {
      const int32_t g = round_bottom(r) + lane;
      ntog = (r < n_rounds && g < batch_top(4 * r)) ? group_table(a, unit, 0, g, 256u, &bad_depth) : 0u;
    }
  };
  auto round_store = [&](int buf) {
#pragma unroll
    for (int i = 0; i < kStagePieces; ++i)
      if (ntake[i]) *reinterpret_cast<uint4 *>(&sym_stage[buf][(lane + 64 * i) * 16]) = nv[i];
    if (ADAPT) table_of_group[buf][lane] = (uint16_t)ntog;
  };
  if (wave == 1) {
    round_load(0);
    round_store(0);
    round_load(1);
  }

  int eslot_feed = 0, eslot_code = 0, eslot_pack = 0, sslot_code = 0, sslot_pack = 0;
  for (int32_t it = 0; it < n_batches + 2; ++it) {
    if (wave == 1) {
      // ---- feeder: entries of batch `it`
      if (it < n_batches) {
        const int32_t r = it >> 2;
        if ((it & 3) == 0 && it > 0) {  // first batch of a new round: land it, start the one after
          round_store(r & 1);
          round_load(r + 1);
        }
        const int32_t top = batch_top(it), bottom = round_bottom(r);
        const uint8_t *sb = sym_stage[r & 1];
        // lane (half h, l) serves step 2p + h of the batch: group top - 1 - 2p - h, rANS lane l
        const int half = lane >> 5, l = lane & 31;
        uint4 *eo = &entry_ring[eslot_feed][half][l];
        if (it > 0) {
          // 16 full groups: all symbol reads, then all table reads, then all ring writes, so that the LDS
          // round trips overlap instead of queueing one behind the other
          const uint8_t *s0 = sb + ((top - bottom - 2 * (kBatch / 2 - 1) - 1 - half) * kLanes + l + (int32_t)mis);
          uint32_t sy[kBatch / 2];
          u32x4 e[kBatch / 2];  // native vectors: each entry moves as one 16-byte LDS access
#pragma unroll
          for (int p = 0; p < kBatch / 2; ++p) sy[p] = s0[2 * kLanes * (kBatch / 2 - 1 - p)];
          if (ADAPT) {  // the group of step 2p + half sits at top - bottom - 1 - half - 2p of the round
            const uint16_t *tg = &table_of_group[r & 1][top - bottom - 2 * (kBatch / 2 - 1) - 1 - half];
#pragma unroll
            for (int p = 0; p < kBatch / 2; ++p) sy[p] += tg[2 * (kBatch / 2 - 1 - p)];
          }
#pragma unroll
          for (int p = 0; p < kBatch / 2; ++p) e[p] = *reinterpret_cast<const u32x4 *>(&table[sy[p]]);
          uint32_t any = 0;
#pragma unroll
          for (int p = 0; p < kBatch / 2; ++p) {
            any |= e[p].w;
            *reinterpret_cast<u32x4 *>(eo + 2 * p * kLanes) = e[p];
          }
          bad_symbol = bad_symbol || (any & 0x80000000u) != 0;
        } else {
          // the top batch: `head` groups, the first of them possibly ragged, then identity steps
#pragma unroll
          for (int p = 0; p < kBatch / 2; ++p) {
            const int j = 2 * p + half;
            const int64_t t = (int64_t)(top - 1 - j) * kLanes + l;
            const bool has = j < head && t < (int64_t)len;
            const int64_t idx = has ? t - (int64_t)bottom * kLanes + mis : 0;
            uint32_t byte = sb[idx];
            if (ADAPT && has) byte += table_of_group[r & 1][top - 1 - j - bottom];
            const uint4 e = table[has ? byte : (uint32_t)kIdentity];
            bad_symbol = bad_symbol || (e.w & 0x80000000u) != 0;
            eo[2 * p * kLanes] = e;
          }
        }
        eslot_feed = eslot_feed == kEntrySlots - 1 ? 0 : eslot_feed + 1;
      }
    } else if (wave == 0) {
      // ---- coder: batch `it - 1`
      if (it >= 1 && it <= n_batches) {
        const uint4 *eb = &entry_ring[eslot_code][0][lane & 31];
        uint32_t *xb = &state_ring[sslot_code][0][lane & 31];
        if (long_form) {
          pipe_batch<true>(x, eb, xb);
        } else {
          pipe_batch<false>(x, eb, xb);
        }
        eslot_code = eslot_code == kEntrySlots - 1 ? 0 : eslot_code + 1;
        sslot_code ^= 1;
      }
    } else {
      // ---- packer: batch `it - 2`
      if (it >= 2) {
        uint32_t top_fill = fill;  // uniform
        // hardware lane h of a half carries rANS lane 31 - h, which the encoder visits first
        const uint32_t *xs = &state_ring[sslot_pack][lane >> 5][31 - (lane & 31)];
        const uint32_t *ts = &entry_ring[eslot_pack][lane >> 5][31 - (lane & 31)].y;
        // In phases, each over all eight step pairs, so that the instructions of a phase do not wait for one
        // another (a lone wavefront waits out the latency of every dependent instruction): reads, emit
        // masks, ranks, list positions, stores.  A lane without a word stores into a slot of its own
        // behind the list instead of sitting out the store.
        uint32_t xps[kBatch / 2], thrs[kBatch / 2], rank[kBatch / 2], base[kBatch / 2];
        uint64_t mask[kBatch / 2];
#pragma unroll
        for (int p = 0; p < kBatch / 2; ++p) {
          xps[p] = xs[2 * p * kLanes];
          thrs[p] = ts[2 * p * kLanes * 4];
        }
#pragma unroll
        for (int p = 0; p < kBatch / 2; ++p) mask[p] = __ballot(xps[p] > thrs[p]);
#pragma unroll
        for (int p = 0; p < kBatch / 2; ++p)
          rank[p] = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask[p] >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask[p], 0u));
#pragma unroll
        for (int p = 0; p < kBatch / 2; ++p) {
          base[p] = top_fill;
          top_fill += (uint32_t)__builtin_popcountll(mask[p]);
        }
#pragma unroll
        for (int p = 0; p < kBatch / 2; ++p) {
          const bool emit = xps[p] > thrs[p];
          word_stage[emit ? base[p] + rank[p] : (uint32_t)(2 * kBatchSyms + 8) + (uint32_t)lane] = (uint16_t)xps[p];
        }
        eslot_pack = eslot_pack == kEntrySlots - 1 ? 0 : eslot_pack + 1;
        sslot_pack ^= 1;
        fill = __builtin_amdgcn_readfirstlane(top_fill);
        // Every second batch (the list holds two batches' words) the complete 16-byte pieces leave, up
        // to two per lane, and the incomplete tail moves to the front.
        if ((it & 1) || it == n_batches + 1) {
          wave_sync();
          const uint32_t full = fill / 8;  // at most 129 pieces
          const bool plain = vbase >= pad && vbase + 8 * full - pad <= cap;
          if (plain) {
            uint16_t *dst = wp + (vbase - pad);  // 16-byte aligned
#pragma unroll
            for (int h = 0; h < 2; ++h)
              if ((uint32_t)(lane + 64 * h) < full)
                *reinterpret_cast<uint4 *>(dst + 8 * (lane + 64 * h)) =
                    *reinterpret_cast<const uint4 *>(word_stage + 8 * (lane + 64 * h));
            if (full > 128 && lane == 0)
              *reinterpret_cast<uint4 *>(dst + 8 * 128) = *reinterpret_cast<const uint4 *>(word_stage + 8 * 128);
          } else {
            for (uint32_t q = lane; q < 8 * full; q += 64) {
              const uint32_t v = vbase + q;
              if (v >= pad && v - pad < cap) wp[v - pad] = word_stage[q];
            }
          }
          const uint32_t rest = fill - 8 * full;
          uint16_t carry = 0;
          if ((uint32_t)lane < rest) carry = word_stage[8 * full + lane];
          wave_sync();
          if ((uint32_t)lane < rest) word_stage[lane] = carry;
          vbase += 8 * full;
          fill = rest;
          wave_sync();
        }
      }
    }
    __syncthreads();
  }

  if (wave == 0) {
    if (lane < kLanes) a.states_out[unit * kLanes + lane] = x;
  } else if (wave == 1) {
    if (bad_symbol || bad_depth) raise(a.status, PLC_ERR_INVALID);  // a symbol with f = 0, or a bad depth
  } else {
    for (uint32_t q = lane; q < fill; q += 64) {  // the incomplete last piece
      const uint32_t v = vbase + q;
      if (v >= pad && v - pad < cap) wp[v - pad] = word_stage[q];
    }
    const uint32_t n_words = vbase + fill - pad;
    if (lane == 0) {
      a.n_words_out[unit] = n_words;
      if ((uint64_t)n_words > a.word_cap) raise(a.status, PLC_ERR_CAPACITY);
    }
  }
}

// ---------------------------------------------------------------------------
// Decoder
// ---------------------------------------------------------------------------
// Slot table: for each of the 4096 slots, sym | (f - 1) << 8 | (slot - cum) << 20.
// Words are consumed from the end of the unit's list.  They are staged through
// a per-wavefront LDS ring of four 512-word blocks (blocks aligned in absolute
// address), refilled at most one block per batch of 16 groups, which consumes
// at most 512 words.  The ring is stored backwards -- word i sits at position
// (~i) mod 2048 -- so that the word of the lane with rank r is at position
// q + r, where q = (-ptr) mod 2048 at the start of a batch and then simply
// grows by the words consumed, in a scalar register; positions 0..543 are
// mirrored at 2048..2591 so that q + r never needs a wrap inside a batch.
constexpr int kRingWords = 2048, kBlockWords = 512, kRingMirror = kBlockWords + 32;

// COMPACT: the slot table is split in two, slot -> symbol (one byte per slot) and symbol -> f - 1 | cum << 16,
// 5 KB instead of 16 KB per table at the price of a second dependent lookup.
constexpr uint32_t kCompactTable = 256 + kScale / 4;  // in 32-bit words
template <bool MASKED, bool COMPACT = false>
__device__ __forceinline__ void dec_step(uint32_t &x, const uint32_t *lut, const uint16_t *&top, uint8_t *sym_slot,
                                         uint32_t below, bool on, uint32_t table_off = 0) {
  uint32_t e;
  if (COMPACT) {
    const uint32_t slot = x & (kScale - 1);
    const uint32_t *mine = lut + table_off;
    const uint32_t s = reinterpret_cast<const uint8_t *>(mine + 256)[slot];
    const uint32_t fc = mine[s];
    e = s | ((fc & 0xfffu) << 8) | ((slot - (fc >> 16)) << 20);
  } else {
    e = lut[(x & (kScale - 1)) + table_off];
  }
  const uint32_t xh = x >> kScaleBits;
  uint32_t xn = __umul24((e >> 8) & 0xfffu, xh) + (xh + (e >> 20));  // f * (x >> 12) + slot - cum
  uint32_t m32 = (uint32_t)__builtin_amdgcn_uicmp(xn, kLow, 36 /* unsigned < */);
  bool need = xn < kLow;
  if (MASKED) {
    need = need && on;
    m32 = (uint32_t)__builtin_amdgcn_ballot_w64(need);
  }
  if (need) {
    // The decoder visits lane 0 first: a lane's word is the rank-th from the top of the list (`top`
    // points at the top word in the backwards ring).  `below` is the mask of the lanes under this one
    // within its half, so that a mirror lane ranks like its twin.
    xn = (xn << 16) | top[__builtin_popcount(m32 & below)];
  }
  top += __builtin_popcount(m32);
  if (MASKED) {
    if (on) {
      *sym_slot = (uint8_t)e;
      x = xn;
    }
  } else {
    *sym_slot = (uint8_t)e;
    x = xn;
  }
}

template <int W, bool ADAPT, bool COMPACT = false>
__global__ __launch_bounds__(W * 64) void rans_decode_kernel(const RansArgs a) {
  __shared__ uint32_t lut_one[ADAPT ? 1 : (COMPACT ? kCompactTable : kScale)];
  extern __shared__ uint32_t lut_per_depth[];  // ADAPT: n_tables slot tables, sized at launch
  uint32_t *lut = ADAPT ? lut_per_depth : lut_one;
  __shared__ uint16_t table_of_group[ADAPT ? W : 1][2][kBatch];  // ADAPT: table offset of each group of a batch
  __shared__ __attribute__((aligned(16))) uint16_t ring[W][kRingWords + kRingMirror];
  __shared__ __attribute__((aligned(16))) uint8_t sym_stage[W][kBatchSyms];
  __shared__ uint32_t table_ok;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t stream = blockIdx.x / a.wgs_per_stream;
  const int64_t chunk = (int64_t)(blockIdx.x - stream * a.wgs_per_stream) * W + wave;
  const bool live = chunk < a.units_per_stream;
  bool bad = false;

  if (!ADAPT) {  // slot table, built by all wavefronts: symbol s is filled in by wavefront s mod W
    uint32_t f[4], cum;
    const uint32_t total = load_freq4(a.freq + stream * 256, lane, f, &cum);
    if (threadIdx.x == 0) table_ok = total == kScale;
    if (total == kScale) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int s = lane * 4 + r;
        if ((s & (W - 1)) == wave) {
          if (COMPACT) {
            lut[s] = ((f[r] - 1u) & 0xfffu) | (cum << 16);  // a symbol that does not occur is never looked up
            for (uint32_t o = 0; o < f[r]; ++o) reinterpret_cast<uint8_t *>(lut + 256)[cum + o] = (uint8_t)s;
          } else {
            for (uint32_t o = 0; o < f[r]; ++o) lut[cum + o] = (uint32_t)s | ((f[r] - 1u) << 8) | (o << 20);
          }
        }
        cum += f[r];
      }
    }
  } else {  // one slot table per bit depth; the table of a depth the stream does not use is all zero
    bool ok = true;
    for (int t = 0; t < a.n_tables; ++t) {
      uint32_t f[4], cum;
      const uint32_t total = load_freq4(a.freq + (stream * a.n_tables + t) * 256, lane, f, &cum);
      ok = ok && (total == kScale || total == 0);
      uint32_t *lt = lut + t * (COMPACT ? kCompactTable : (uint32_t)kScale);
      if (total == kScale) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int s = lane * 4 + r;
          if ((s & (W - 1)) == wave) {
            if (COMPACT) {
              lt[s] = ((f[r] - 1u) & 0xfffu) | (cum << 16);
              for (uint32_t o = 0; o < f[r]; ++o) reinterpret_cast<uint8_t *>(lt + 256)[cum + o] = (uint8_t)s;
            } else {
              for (uint32_t o = 0; o < f[r]; ++o) lt[cum + o] = (uint32_t)s | ((f[r] - 1u) << 8) | (o << 20);
            }
          }
          cum += f[r];
        }
      } else {
        for (uint32_t o = threadIdx.x; o < (COMPACT ? kCompactTable : (uint32_t)kScale); o += W * 64) lt[o] = 0u;
      }
    }
    if (threadIdx.x == 0) table_ok = ok;
  }
  __syncthreads();
  if (!table_ok) {  // not a table: nothing can be decoded
    if (live && lane == 0) raise(a.status, PLC_ERR_CORRUPT);
    return;
  }
  if (!live) return;  // no workgroup barrier below

  const int64_t unit = stream * a.units_per_stream + chunk;
  const int64_t begin = chunk * a.unit_syms;
  const int64_t rest = a.syms_per_stream - begin;
  const uint32_t len = (uint32_t)(rest < a.unit_syms ? rest : a.unit_syms);
  uint8_t *ubase = a.sym_out + stream * a.syms_per_stream + begin;
  const bool out_aligned = (reinterpret_cast<uintptr_t>(ubase) & 15u) == 0;
  const int32_t G = (int32_t)((len + kLanes - 1) / kLanes);
  const uint32_t top_syms = len - (uint32_t)(G - 1) * kLanes;

  // ---- word list geometry, relative to a 1 KiB-aligned address at or below the unit's first word
  const uint64_t off = a.word_off[unit];
  const uint32_t n = a.n_words_in[unit];
  if (off > a.words_len || (uint64_t)n > a.words_len - off) {
    if (lane == 0) raise(a.status, PLC_ERR_CORRUPT);
    return;
  }
  const uint16_t *first_word = a.words_in + off;
  const int32_t lo = (int32_t)((reinterpret_cast<uintptr_t>(first_word) & (uintptr_t)(kBlockWords * 2 - 1)) >> 1);
  const uint16_t *aligned_base = first_word - lo;  // pointer arithmetic keeps the loads global, not flat
  const int32_t hi = lo + (int32_t)n;
  uint16_t *myring = ring[wave];

  // one 16-byte piece (eight words) of block blk per lane, if the piece holds a word of this unit
  auto block_load = [&](int32_t blk, uint4 &v) -> bool {
    const int32_t first = blk * kBlockWords + lane * 8;
    const bool take = blk >= 0 && hi > lo && first + 8 > lo && first < hi;
    if (take) v = *reinterpret_cast<const uint4 *>(aligned_base + first);
    return take;
  };
  // word i goes to ring position (~i) mod 2048: a piece of eight words lands reversed on an aligned run
  auto block_store = [&](int32_t blk, bool take, const uint4 &v) {
    if (take) {
      const uint32_t pos = (uint32_t)(~(blk * kBlockWords + lane * 8 + 7)) & (kRingWords - 1);
      const uint4 r = make_uint4((v.w >> 16) | (v.w << 16), (v.z >> 16) | (v.z << 16), (v.y >> 16) | (v.y << 16),
                                 (v.x >> 16) | (v.x << 16));
      *reinterpret_cast<uint4 *>(myring + pos) = r;
      if (pos < kRingMirror) *reinterpret_cast<uint4 *>(myring + kRingWords + pos) = r;
    }
  };

  int32_t ptr = hi;
  int32_t lowest = ((hi - 1) >> 9) + 1;  // lowest block already staged (none yet)
  for (int r = 0; r < 2; ++r) {          // the two top blocks
    uint4 v;
    const int32_t blk = lowest - 1;
    const bool take = block_load(blk, v);
    block_store(blk, take, v);
    lowest = blk;
  }
  wave_sync();

  const bool coder = lane < kLanes;
  const int rl = lane & (kLanes - 1);
  const uint32_t below = (1u << rl) - 1u;
  const bool top_active = (uint32_t)rl < top_syms;
  uint32_t x = a.states_in[unit * kLanes + rl];

  // Full batches of 16 groups are fully unrolled; the groups that do not fill a batch (and the last
  // group if it is ragged) form a tail that runs in a rolled loop.
  int32_t tail_groups = G % kBatch;
  if (tail_groups == 0 && top_syms < kLanes) tail_groups = kBatch;
  const int32_t g_tail = G - tail_groups;
  uint8_t *sb = &sym_stage[wave][rl];

  // ADAPT: table offsets of the batch's 16 groups, fetched one batch ahead by lanes 0..15
  bool bad_depth = false;
  auto group_load = [&](int32_t g0) -> uint32_t {
    const int32_t g = g0 + lane;
    if (!ADAPT || lane >= kBatch || g >= G) return 0u;
    return group_table(a, stream, begin, g, COMPACT ? kCompactTable : (uint32_t)kScale, &bad_depth);
  };
  if (ADAPT) {
    const uint32_t gt0 = group_load(0);
    if (lane < kBatch) table_of_group[wave][0][lane] = (uint16_t)gt0;
    wave_sync();
  }
  int gbuf = 0;

  for (int32_t g0 = 0; g0 < G; g0 += kBatch) {
    const bool tail = g0 >= g_tail;
    const int32_t cnt_groups = tail ? tail_groups : kBatch;
    // stage one more block below if the coming batches may reach it
    const int32_t top = (ptr - 1) >> 9;
    const bool fetch = lowest > top - 2;
    const int32_t blk = lowest - 1;
    uint4 pre;
    bool ptake = false;
    if (fetch) ptake = block_load(blk, pre);
    const uint32_t ngt = group_load(g0 + kBatch);
    const uint16_t *gt = table_of_group[ADAPT ? wave : 0][gbuf];

    const uint16_t *wtop0 = myring + ((uint32_t)(-ptr) & (kRingWords - 1));
    const uint16_t *wtop = wtop0;
    if (tail) {
      for (int32_t j = 0; j < cnt_groups; ++j)
        dec_step<true, COMPACT>(x, lut, wtop, sb + kLanes * j, below, j != cnt_groups - 1 || top_active,
                                ADAPT ? gt[j] : 0u);
    } else {
      // the batch's table offsets are read before its first symbol is stored (the compiler cannot tell
      // the two LDS arrays apart, and a read inside a step would queue behind the previous step's store)
      uint32_t off[kBatch];
#pragma unroll
      for (int j = 0; j < kBatch; ++j) off[j] = ADAPT ? (uint32_t)__builtin_amdgcn_readfirstlane(gt[j]) : 0u;
#pragma unroll
      for (int j = 0; j < kBatch; ++j) dec_step<false, COMPACT>(x, lut, wtop, sb + kLanes * j, below, true, off[j]);
    }
    if (ADAPT) {
      if (lane < kBatch) table_of_group[wave][gbuf ^ 1][lane] = (uint16_t)ngt;
      gbuf ^= 1;
    }
    ptr -= (int32_t)(wtop - wtop0);
    if (ptr < lo) {  // ran out of words: the stream is damaged
      bad = true;
      ptr = lo;
    }
    // the prefetched block goes to the ring BEFORE this batch's symbols are stored: waiting for the load
    // then does not also wait for freshly issued stores (loads and stores share one counter)
    if (fetch) {
      block_store(blk, ptake, pre);
      lowest = blk;
    }
    wave_sync();
    // drain the batch's symbols
    const uint32_t done = (uint32_t)g0 * kLanes;
    const uint32_t room = (uint32_t)cnt_groups * kLanes;
    const uint32_t nsym = (len - done) < room ? (len - done) : room;
    if (out_aligned) {
      const uint32_t full = nsym / 16;
      if ((uint32_t)lane < full)
        *reinterpret_cast<uint4 *>(ubase + done + lane * 16) =
            *reinterpret_cast<const uint4 *>(&sym_stage[wave][lane * 16]);
      const uint32_t tail = full * 16 + (uint32_t)lane;
      if (tail < nsym) ubase[done + tail] = sym_stage[wave][tail];
    } else {
      for (uint32_t i = lane; i < nsym; i += 64) ubase[done + i] = sym_stage[wave][i];
    }
    wave_sync();
  }
  // integrity: every word consumed, every lane back at the initial state
  if (ptr != lo || (coder && x != kLow)) bad = true;
  if (bad) raise(a.status, PLC_ERR_CORRUPT);
  if (bad_depth) raise(a.status, PLC_ERR_INVALID);
}

// ---------------------------------------------------------------------------
// Reconstruction inside the decoder for units coded as whole streams
// ---------------------------------------------------------------------------
// A further wavefront of the unit's workgroup that turns each batch of decoded symbols into KV components
// while the next batches are decoded: out = prediction over RK candidates + symbol * step (the arithmetic
// of plc_reconstruct; COND: of plc_reconstruct_cond; ADAPT: of plc_reconstruct_adapt).  A batch is 512 symbols = 64 chunks of 8 components,
// one chunk per lane.  The candidates and weights of a chunk do not depend on its symbols, so they are
// requested kRecDepth batches ahead (a template parameter) and are in registers when the symbols arrive.  The wavefront meets the
// decoder at every batch barrier -- one "start" barrier, then one per batch, in step with the other
// wavefronts of the workgroup -- through the bare instruction, which unlike __syncthreads does not first
// wait for its outstanding loads.  Loads are issued by every lane in every batch (past the end of the stream
// a lane stays on its last chunk and stores nothing), so that the number of loads behind any given one is the
// same on every path and the wait before a use leaves the later requests in flight (the few loads and
// stores that escapes add are issued only where there are escapes and cost at most their own number in
// that count).
//   stream, len, G   the unit's stream, its symbols and groups of 32
//   sym_stage        the two symbol stages: batch b is in stage b mod 2 from its barrier to the next (kLate = 1:
//                    from the barrier after its own, where the symbols pass through another wavefront first)
constexpr int kRecDepthBase = 3;  // batches a request runs ahead of its symbols

template <int RK, bool COND, bool ADAPT, int kRecDepth, int kLate = 0, int kStageSyms = 2 * kBatchSyms>
__device__ __forceinline__ void reconstruct_batches(const RansArgs &a, int64_t stream, uint32_t len, int32_t G,
                                                    const uint8_t (&sym_stage)[2][kStageSyms], int lane) {
  static_assert(COND || !ADAPT, "the adaptive quantiser lives on the token-conditional path");
  const ReconView &r = a.recon;
  const uint32_t lh = (uint32_t)(r.L * r.H);
  const uint32_t s = (uint32_t)stream / lh, rem = (uint32_t)stream - s * lh;
  const uint32_t l = rem / (uint32_t)r.H, h = rem - l * (uint32_t)r.H;
  const int64_t cand0 = s * r.cs[0] + l * r.cs[1] + h * r.cs[2];
  const int64_t out0 = s * r.as[0] + l * r.as[1] + h * r.as[2];
  const float *w0 = r.weights + (int64_t)s * r.n * r.k;
  const uint32_t n_chunks = len / kChunk;
  const uint32_t d8 = (uint32_t)r.d8, adv_row = 64u / d8, adv_e8 = 64u - adv_row * d8;
  // The chunk this lane requests next: row = position * 2 + (0 = K, 1 = V), e8 = chunk inside the row,
  // and where its candidates, weights and output are.  From batch to batch a lane moves on by 64
  // chunks; where that is a whole, even number of rows (d = 8, 16, ... 256) it is the same position
  // step in the same half every time, and the three pointers advance by constants.
  uint32_t at_chunk = (uint32_t)lane, row = (uint32_t)lane / d8, e8 = (uint32_t)lane - row * d8;
  const bool steady = adv_e8 == 0u && (adv_row & 1u) == 0u;
  const int64_t cand_step = (int64_t)(adv_row / 2u) * r.cs[3], out_step = (int64_t)(adv_row / 2u) * r.as[3];
  const uint32_t w_step = (adv_row / 2u) * (uint32_t)RK;
  const uint16_t *cand_p;
  const float *w_p;
  uint16_t *out_p;
  auto point = [&](uint32_t rr, uint32_t ee) {
    const uint32_t i = rr >> 1;
    cand_p = ((rr & 1u) ? r.cand_v : r.cand_k) + cand0 + (int64_t)i * r.cs[3] + ee * kChunk;
    w_p = w0 + (int64_t)i * RK;
    out_p = ((rr & 1u) ? r.out_v : r.out_k) + out0 + (int64_t)i * r.as[3] + ee * kChunk;
  };
  if (at_chunk < n_chunks) {
    point(row, e8);
  } else {
    point(0u, 0u);
  }
  // COND: the position names its true candidate (plc_reconstruct_cond), whose vector then is the
  // prediction; which candidate to request is itself a load, so it runs one round further ahead: a
  // second cursor walks the chunks 2 * kRecDepth batches in front and fetches their chosen index.
  // ADAPT: the position's bit depth, which sets its step, is fetched with the chosen index.
  uint32_t far_chunk = at_chunk, far_row = row, far_e8 = e8;
  int64_t far_pos = (int64_t)s * r.n + (at_chunk < n_chunks ? row >> 1 : 0u);  // entry in chosen and bits
  int32_t pick_next[kRecDepth];  // chosen index of the chunk the stage requests next
  int32_t pick_used[kRecDepth];  // and of the chunk whose candidates it holds (-1: the weighted mean)
  bool mean_path[kRecDepth];     // uniform: some lane of the stage's request needed all candidates
  uint32_t depth_next[kRecDepth], depth_used[kRecDepth];  // bit depths, the same way
  uint4 cv[kRecDepth][RK];
  float wv[kRecDepth][RK];
  typedef __attribute__((address_space(1))) u32x4 *global_u32x4;  // named global: kept through the loop
  global_u32x4 dst[kRecDepth];
  bool live[kRecDepth];  // whether the lane's chunk exists (a flag of its own: the pointer stays a global one)
  // Escapes.  This wavefront sees every chunk of the stream in order, so the number of escapes in front
  // of a chunk is a running count plus a prefix over the lanes.  A chunk with escapes is not stored when
  // its symbols arrive: its raw values are requested from the stream's list, the chunk is held, and the
  // next time the same registers come round, kRecDepth batches later, the values that have arrived are
  // put over its escaped components and the chunk is stored, once and whole.  The registers hold up to
  // kEscLate raw values per chunk; a batch in which some chunk has more (3e-5 of the chunks at the synthetic
  // workloads' escape rates) fetches its raw values, waits for them and stores its escaped chunks at once.
  constexpr int kEscLate = 2;
  uint32_t esc_bits[kRecDepth];  // which components of the chunk held for esc_dst await their raw value
  uint32_t esc_raw[kRecDepth][kEscLate];
  u32x4 esc_held[kRecDepth];
  global_u32x4 esc_dst[kRecDepth];
  const uint64_t esc_base = r.esc_off[stream];
  uint32_t esc_seen = 0;  // escapes of the stream so far
#pragma unroll
  for (int j = 0; j < kRecDepth; ++j) esc_bits[j] = 0u, esc_dst[j] = nullptr, esc_held[j] = u32x4{0u, 0u, 0u, 0u};
  // Loads of the lane's next chunk (of its last one again once the stream is at its end, so that every
  // batch issues the same loads), then on to the chunk after it.
  auto load_weights = [&](float(&w)[RK]) {
    if constexpr (RK % 4 == 0) {
#pragma unroll
      for (int j = 0; j < RK; j += 4) {
        const float4 t = *reinterpret_cast<const float4 *>(w_p + j);
        w[j] = t.x, w[j + 1] = t.y, w[j + 2] = t.z, w[j + 3] = t.w;
      }
    } else {
#pragma unroll
      for (int j = 0; j < RK; ++j) w[j] = w_p[j];
    }
  };
  auto fetch_pick = [&](int32_t &pick, uint32_t &depth) {  // COND: the far cursor's position, then one batch on
    pick = r.chosen[far_pos];
    if constexpr (ADAPT) depth = r.bits[far_pos];
    far_chunk += 64u;
    if (steady) {  // uniform
      if (far_chunk < n_chunks) far_pos += adv_row / 2u;
    } else {
      far_row += adv_row;
      far_e8 += adv_e8;
      if (far_e8 >= d8) {
        far_e8 -= d8;
        ++far_row;
      }
      if (far_chunk < n_chunks) far_pos = (int64_t)s * r.n + (far_row >> 1);
    }
  };
  auto request = [&](uint4(&c)[RK], float(&w)[RK], global_u32x4 &out, bool &ok, int32_t &pick_nx,
                     int32_t &pick_us, bool &mean, uint32_t &depth_nx, uint32_t &depth_us) {
    if constexpr (COND) {
      int32_t pick = pick_nx;
      if (pick < -1 || pick >= RK) {
        raise(a.status, PLC_ERR_INVALID);
        pick = -1;
      }
      if constexpr (ADAPT) {
        uint32_t b = depth_nx;
        if (b < 1u || b > (uint32_t)PLC_MAX_BITS) {
          raise(a.status, PLC_ERR_INVALID);
          b = 1u;
        }
        depth_us = b;
      }
      mean = __ballot(pick < 0) != 0;  // uniform
      if (!mean) {
        c[0] = load16_stream(cand_p + pick * r.cs[4]);
      } else {  // a lane that has its candidate takes it RK times: every lane issues the same loads
#pragma unroll
        for (int j = 0; j < RK; ++j) c[j] = load16_stream(cand_p + (pick >= 0 ? pick : j) * r.cs[4]);
        load_weights(w);
      }
      pick_us = pick;
      fetch_pick(pick_nx, depth_nx);
    } else {
#pragma unroll
      for (int j = 0; j < RK; ++j) c[j] = load16_stream(cand_p + j * r.cs[4]);
      load_weights(w);
    }
    out = (global_u32x4)out_p;
    ok = at_chunk < n_chunks;
    at_chunk += 64u;
    if (steady) {  // uniform
      if (at_chunk < n_chunks) cand_p += cand_step, w_p += w_step, out_p += out_step;
    } else {
      row += adv_row;
      e8 += adv_e8;
      if (e8 >= d8) {
        e8 -= d8;
        ++row;
      }
      if (at_chunk < n_chunks) point(row, e8);
    }
  };
  // the raw values that have arrived for the chunk held for `out`: over its escaped components, lowest
  // first (component e is half e & 1 of word e >> 1), then the chunk goes out
  // one raw value over the lowest component still marked in `bits`
  auto put_raw = [](u32x4 &chunk, uint32_t &bits, uint32_t raw) {
    const uint32_t e = (uint32_t)__builtin_ctz(bits);
    bits &= bits - 1u;
    const uint32_t shift = (e & 1u) * 16u, keep = ~(0xffffu << shift), value = (raw & 0xffffu) << shift;
#pragma unroll
    for (uint32_t word = 0; word < 4; ++word)
      chunk[word] = (e >> 1) == word ? (chunk[word] & keep) | value : chunk[word];
  };
  auto patch = [&](global_u32x4 out, uint32_t &bits, const uint32_t (&raw)[kEscLate], u32x4 &held) {
    if (__ballot(bits != 0u) == 0) return;  // uniform
    const bool pending = bits != 0u;
#pragma unroll
    for (int i = 0; i < kEscLate; ++i) {
      if (i > 0 && __ballot(bits != 0u) == 0) break;  // uniform; seldom more than one per chunk
      if (bits) put_raw(held, bits, raw[i]);
    }
    if (pending) __builtin_nontemporal_store(held, out);
  };
  if constexpr (COND) {
#pragma unroll
    for (int j = 0; j < kRecDepth; ++j) fetch_pick(pick_next[j], depth_next[j]);
  }
#pragma unroll
  for (int j = 0; j < kRecDepth; ++j)
    request(cv[j], wv[j], dst[j], live[j], pick_next[j], pick_used[j], mean_path[j], depth_next[j], depth_used[j]);
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();  // barrier "start"
  asm volatile("" ::: "memory");
  if constexpr (kLate > 0) {  // the first batch's own barrier: its symbols come one barrier later
    static_assert(kLate == 1, "one barrier behind");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  }
  const int32_t n_batches = (G + kBatch - 1) / kBatch;
  const int32_t n_full = (int32_t)(n_chunks / 64u);  // batches all of whose chunks exist
  // One batch: join its barrier, take its symbols from the stage, finish the chunk, request the chunk
  // of the batch kRecDepth later into the registers just freed.
  auto turn = [&](uint4(&c)[RK], float(&w)[RK], global_u32x4 &out, bool &ok, uint32_t &bits,
                  uint32_t(&raw)[kEscLate], u32x4 &held, global_u32x4 &late, int32_t &pick_nx, int32_t &pick_us, bool &mean,
                  uint32_t &depth_nx, uint32_t &depth_us, int32_t b, bool whole) {
    // (the scheduler would otherwise start on the predictions of all kRecDepth batches at the top of a
    // pass, and so wait there for requests that have only just gone out)
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();  // barrier of batch b (kLate: the one after): its symbols are in the stage
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    const uint2 sv = *reinterpret_cast<const uint2 *>(&sym_stage[b & 1][lane * kChunk]);
    patch(late, bits, raw, held);
    float pred[kChunk];
    if (!COND || mean) {  // uniform
#pragma unroll
      for (int e = 0; e < kChunk; ++e) pred[e] = 0.0f;
#pragma unroll
      for (int j = 0; j < RK; ++j) accumulate8(w[j], c[j], pred);
    }
    if constexpr (COND) {
      const half8 own = __builtin_bit_cast(half8, c[0]);
#pragma unroll
      for (int e = 0; e < kChunk; ++e) pred[e] = (!mean || pick_us >= 0) ? (float)own[e] : pred[e];
    }
    uint32_t unused = 0;
    const float step = ADAPT ? __builtin_ldexpf(r.range, -(int)depth_us) : r.delta;
    const half8 v = add_back8(sv, step, pred, &unused);
    const bool mine = whole || ok;
    // a byte is 0xff iff its low seven bits carry into bit 7 when 1 is added and bit 7 is set
    const uint32_t hx = ((sv.x & 0x7f7f7f7fu) + 0x01010101u) & sv.x & 0x80808080u;
    const uint32_t hy = ((sv.y & 0x7f7f7f7fu) + 0x01010101u) & sv.y & 0x80808080u;
    const bool has = mine && (hx | hy) != 0u;
    if (mine && !has) __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v), out);
    const uint64_t lanes = __ballot(has);
    if (lanes != 0) {  // uniform
      // bit 7 of byte e to bit e
      const uint32_t mx = ((hx >> 7) * 0x00204081u) >> 21 & 0xfu, my = ((hy >> 7) * 0x00204081u) >> 21 & 0xfu;
      bits = has ? (mx | (my << 4)) : 0u;
      const uint32_t n_esc = (uint32_t)__builtin_popcount(bits);
      const bool several = __ballot(n_esc > 1u) != 0;  // uniform; seldom
      uint32_t total, before;
      if (!several) {
        before = __builtin_amdgcn_mbcnt_hi((uint32_t)(lanes >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)lanes, 0u));
        total = (uint32_t)__builtin_popcountll(lanes);
      } else {
        before = wave_escape_prefix(n_esc, &total);
      }
      const uint64_t src = esc_base + esc_seen + before;
      esc_seen += total;
      if (several && __ballot(n_esc > (uint32_t)kEscLate) != 0) {  // uniform; rare: fetch, wait, store now
        u32x4 now = __builtin_bit_cast(u32x4, v);
#pragma unroll
        for (int i = 0; i < kChunk; ++i) {
          if (__ballot(bits != 0u) == 0) break;  // uniform
          if (bits) {
            uint32_t value = 0u;
            if (src + i < r.esc_len) {
              value = r.esc_in[src + i];
            } else {
              raise(a.status, PLC_ERR_CORRUPT);
            }
            put_raw(now, bits, value);
          }
        }
        if (has) __builtin_nontemporal_store(now, out);  // bits is 0 again: nothing is held
      } else {
        held = __builtin_bit_cast(u32x4, v);
        late = out;
#pragma unroll
        for (int i = 0; i < kEscLate; ++i) {
          if (i > 0 && (!several || __ballot(n_esc > (uint32_t)i) == 0)) break;  // uniform
          if (n_esc > (uint32_t)i) {
            if (src + i < r.esc_len) {
              raw[i] = r.esc_in[src + i];
            } else {
              raise(a.status, PLC_ERR_CORRUPT);
              raw[i] = 0u;
            }
          }
        }
      }
    }
    request(c, w, out, ok, pick_nx, pick_us, mean, depth_nx, depth_us);
  };
  // Whole batches, kRecDepth at a time and free of branches: every pass issues the same loads and
  // stores in the same order.
  int32_t b0 = 0;
  for (; b0 + kRecDepth <= n_full; b0 += kRecDepth) {
#pragma unroll
    for (int j = 0; j < kRecDepth; ++j)
      turn(cv[j], wv[j], dst[j], live[j], esc_bits[j], esc_raw[j], esc_held[j], esc_dst[j], pick_next[j], pick_used[j],
           mean_path[j], depth_next[j], depth_used[j], b0 + j, true);
  }
  // What is left: fewer than kRecDepth whole batches and possibly a partial one.
#pragma unroll
  for (int j = 0; j < kRecDepth; ++j)
    if (b0 + j < n_batches)  // uniform
      turn(cv[j], wv[j], dst[j], live[j], esc_bits[j], esc_raw[j], esc_held[j], esc_dst[j], pick_next[j], pick_used[j],
           mean_path[j], depth_next[j], depth_used[j], b0 + j, false);
#pragma unroll
  for (int j = 0; j < kRecDepth; ++j) patch(esc_dst[j], esc_bits[j], esc_raw[j], esc_held[j]);
}

// ---------------------------------------------------------------------------
// Decoder for streams coded as one unit (one wavefront per workgroup)
// ---------------------------------------------------------------------------
// With one unit per stream there are only as many wavefronts as streams, so what counts is the
// length of the dependent chain of one step: a lone wavefront waits out the full latency of every
// instruction whose result the next one needs (measured: with the table lookup replaced by arithmetic a
// step still took 130 of its 180 cycles).  In the kernel above that chain holds two LDS round trips --
// slot table, then, for the lanes that renormalise, the word -- and some ten dependent vector
// instructions.  Here the round trips are folded into one and the instructions behind it cut to five.
//
// Every entry, of the slot table and of the word ring alike, is 8 bytes
//     .x = f | sym << 24        .y = f * w4 + slot - cum
// A ring entry stands for a word w = w4 << 12 | slot: it is the slot-table entry that the state will
// select once the word has been shifted in (the state's low 12 bits are then the word's, which is all
// they are needed for), with the word's top four bits w4 already multiplied in; in the slot table itself
// w4 = 0.  A lane that renormalises reads its ring entry, a lane that does not reads the slot table at
// its new state -- one read either way, at an address chosen per lane, both tables living in one LDS
// array; the ring entries are formed when a block of words is staged, off the chain.  The state is
// carried as xc = x >> 12 without the bits the word supplies: from the previous step's value v,
// xc = v << 4 if the lane renormalised and v >> 12 if not (ready long before the entry arrives), so
// that f * (x >> 12) + slot - cum = f * (xc + w4) + slot - cum = f * xc + .y: one multiply-add, whose
// 24-bit multiplicand ignores the symbol in the top byte of .x.
// The ring holds RB blocks of 512 words.  Four let the helper leave its newest block on its way for a batch
// (below); three are what the decoder strictly needs -- the block of the pointer, the one below it, and the
// one being staged for the batch after -- and bring the workgroup's LDS from 56.6 to 52.5 KB, so that a
// compute unit holds three workgroups instead of two where the registers allow it (k <= 6).  That is the
// variant for thousands of streams, where units in flight count for more than the helper's wait: 9.1 -> 7.9 ms
// on 5120 streams with k = 4.  (With k = 8 and 16,384 streams the kernel is bound by HBM at 5.4 TB/s whatever
// the workgroups per compute unit or the depth of the reconstruction's requests: two, three or four batches
// ahead, two or three workgroups, all within 0.1 % of one another.)

template <bool MASKED>
__device__ __forceinline__ void dec_chain_step(uint32_t &xc, uint2 &e, const uint2 *tab, uint32_t &ring_at,
                                               uint8_t *sym_slot, bool on) {
  const uint32_t xn = __umul24(e.x, xc) + e.y;  // f * (x >> 12) + slot - cum
  uint32_t m32 = (uint32_t)__builtin_amdgcn_uicmp(xn, kLow, 36 /* unsigned < */);
  bool need = xn < kLow;
  if (MASKED) {
    need = need && on;
    m32 = (uint32_t)__builtin_amdgcn_ballot_w64(need);
  }
  // ring entry of the rank-th word from the top (lane 0 is served first: the rank is the number of
  // renormalising lanes below this one), or slot-table entry of xn
  uint32_t idx_ring = __builtin_amdgcn_mbcnt_lo(m32, ring_at);
  uint32_t idx_slot = xn & (kScale - 1);
  asm volatile("" : "+v"(idx_ring), "+v"(idx_slot));  // both in registers: the choice is one select, not a branch
  const uint2 en = tab[need ? idx_ring : idx_slot];
  __builtin_amdgcn_sched_barrier(0);  // what follows is issued in the shadow of the read
  // (the entry of the top word, uniform, kept in a vector register where the rank is added to it: a count and
  // an add per step)
  ring_at += (uint32_t)__builtin_popcount(m32);
  asm volatile("" : "+v"(ring_at));
  const uint32_t next = need ? (xn << 4) : (xn >> kScaleBits);
  if (!MASKED || on) {
    *sym_slot = (uint8_t)(e.x >> 24);
    xc = next;
    e = en;
  }
}

// Two wavefronts per unit.  What a step does not need stays off the decoding wavefront: a helper, on
// another SIMD of the compute unit, stages the words (forming the ring entries costs eight table lookups
// and up to sixteen LDS writes per lane and block) and moves the decoded symbols to global memory.  The
// two meet at one workgroup barrier per batch of 16 steps:
//   decoder  batch b: 16 steps into symbol stage b % 2; publishes the word pointer; barrier b
//   helper   while batch b runs: stages every block down to 1024 words below the pointer published at
//            barrier b - 1 (a batch consumes at most 512, so batch b + 1 finds its words); barrier b;
//            then moves the symbols of batch b out while batch b + 1 runs.
// The blocks the helper writes lie at least one block below those the running batch reads, and the ring
// slots they take belonged to blocks above the pointer (four blocks of ring: the pointer's block and the
// three below it).
//
// RK > 0 adds a third wavefront that reconstructs the KV components of each batch while the next batches are
// decoded (reconstruct_batches above).
template <int RK, bool COND, int RB = 4>
__global__ __launch_bounds__(RK ? 192 : 128) void rans_decode_chain_kernel(const RansArgs a) {
  static_assert(RB == 3 || RB == 4, "ring blocks");
  constexpr uint32_t kRing = RB * kBlockWords;  // words the ring holds: word i sits at kRing - 1 - i mod kRing
  __shared__ __attribute__((aligned(16))) uint2 tab[kScale + kRing + kRingMirror];  // slot table, then the ring
  __shared__ __attribute__((aligned(16))) uint8_t sym_stage[2][2 * kBatchSyms];  // second half: lanes 32..63
  __shared__ uint32_t fc[256];
  __shared__ int32_t ptr_pub[2];  // the word pointer after batch b, in slot b mod 2
  constexpr int kThreads = RK ? 192 : 128;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const bool helper = wave == 1;
  const int64_t stream = blockIdx.x / a.wgs_per_stream;
  const int64_t chunk = blockIdx.x - stream * a.wgs_per_stream;
  bool bad = false;

  {  // slot table: symbols one after the other, 128 slots per pass
    uint32_t f[4], cum;
    const uint32_t total = load_freq4(a.freq + stream * 256, lane, f, &cum);
    if (total != kScale) {  // not a table: nothing can be decoded (both wavefronts leave, before any barrier)
      if (threadIdx.x == 0) raise(a.status, PLC_ERR_CORRUPT);
      return;
    }
    if (wave == 0) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        fc[lane * 4 + r] = f[r] | (cum << 16);
        cum += f[r];
      }
    }
    __syncthreads();
    for (int s = 0; s < 256; ++s) {
      const uint32_t v = fc[s];
      const uint32_t fs = v & 0xffffu, cs = v >> 16;
      for (uint32_t o = threadIdx.x; o < fs; o += kThreads) tab[cs + o] = make_uint2(fs | ((uint32_t)s << 24), o);
    }
    __syncthreads();
  }
  uint2 *ring = tab + kScale;

  const int64_t unit = stream * a.units_per_stream + chunk;
  const int64_t begin = chunk * a.unit_syms;
  const int64_t rest = a.syms_per_stream - begin;
  const uint32_t len = (uint32_t)(rest < a.unit_syms ? rest : a.unit_syms);
  uint8_t *ubase = a.sym_out + stream * a.syms_per_stream + begin;
  const bool out_aligned = (reinterpret_cast<uintptr_t>(ubase) & 15u) == 0;
  const int32_t G = (int32_t)((len + kLanes - 1) / kLanes);
  const uint32_t top_syms = len - (uint32_t)(G - 1) * kLanes;

  // ---- word list geometry, relative to a 1 KiB-aligned address at or below the unit's first word
  const uint64_t off = a.word_off[unit];
  const uint32_t n = a.n_words_in[unit];
  if (off > a.words_len || (uint64_t)n > a.words_len - off) {  // uniform: both wavefronts leave
    if (threadIdx.x == 0) raise(a.status, PLC_ERR_CORRUPT);
    return;
  }
  const uint16_t *first_word = a.words_in + off;
  const int32_t lo = (int32_t)((reinterpret_cast<uintptr_t>(first_word) & (uintptr_t)(kBlockWords * 2 - 1)) >> 1);
  const uint16_t *aligned_base = first_word - lo;  // pointer arithmetic keeps the loads global, not flat
  const int32_t hi = lo + (int32_t)n;

  int32_t tail_groups = G % kBatch;
  if (tail_groups == 0 && top_syms < kLanes) tail_groups = kBatch;
  const int32_t g_tail = G - tail_groups;

  if constexpr (RK > 0) {
    if (wave == 2) {
      reconstruct_batches<RK, COND, false, kRecDepthBase>(a, stream, len, G, sym_stage, lane);
      return;
    }
  }

  if (helper) {
    // one 16-byte piece (eight words) of block blk per lane, if the piece holds a word of this unit
    auto block_load = [&](int32_t blk, uint4 &v) -> bool {
      const int32_t first = blk * kBlockWords + lane * 8;
      const bool take = blk >= 0 && hi > lo && first + 8 > lo && first < hi;
      if (take) v = *reinterpret_cast<const uint4 *>(aligned_base + first);
      return take;
    };
    // Word i goes to ring position (~i) mod 2048: the slot-table entry of its low 12 bits, its top four
    // bits multiplied in.
    auto block_store = [&](int32_t blk, bool take, const uint4 &v) {
      if (take) {
        // ring position of the piece's last word (blk >= 0 here)
        const uint32_t pos = (RB - 1u - (uint32_t)blk % RB) * kBlockWords + (uint32_t)(kBlockWords - 8 - lane * 8);
        const uint32_t w[8] = {v.x & 0xffffu, v.x >> 16, v.y & 0xffffu, v.y >> 16,
                               v.z & 0xffffu, v.z >> 16, v.w & 0xffffu, v.w >> 16};
        uint2 en[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) en[i] = tab[w[7 - i] & (kScale - 1)];  // en[i] belongs at pos + i
#pragma unroll
        for (int i = 0; i < 8; ++i) en[i].y += __umul24(en[i].x, w[7 - i] >> kScaleBits);  // f * w4 <= 4096 * 15
#pragma unroll
        for (int i = 0; i < 8; i += 2)
          *reinterpret_cast<uint4 *>(&ring[pos + i]) = make_uint4(en[i].x, en[i].y, en[i + 1].x, en[i + 1].y);
        if (pos < (uint32_t)kRingMirror) {
#pragma unroll
          for (int i = 0; i < 8; i += 2)
            *reinterpret_cast<uint4 *>(&ring[kRing + pos + i]) =
                make_uint4(en[i].x, en[i].y, en[i + 1].x, en[i + 1].y);
        }
      }
    };
    // Stages every block that holds a word at or above `down_to` and is not staged yet.  The last of them
    // may be left on its way (`ahead`): its words go to the ring at the next call, a batch later, so that
    // the wavefront does not sit out the load's latency in front of the barrier.
    int32_t lowest = ((hi - 1) >> 9) + 1;  // lowest block already requested (none yet)
    uint4 ahead_v;
    int32_t ahead_blk = 0;
    bool ahead = false, ahead_take = false;
    auto stage_down_to = [&](int32_t down_to, bool leave_one) {
      if (ahead) {  // uniform
        block_store(ahead_blk, ahead_take, ahead_v);
        ahead = false;
      }
      const int32_t last = down_to > 0 ? down_to >> 9 : 0;
      while (lowest > last) {  // uniform; one round per batch after the first call
        const int32_t blk = lowest - 1;
        lowest = blk;
        if (leave_one && blk == last) {
          ahead_take = block_load(blk, ahead_v);
          ahead_blk = blk;
          ahead = true;
        } else {
          uint4 v;
          const bool take = block_load(blk, v);
          block_store(blk, take, v);
        }
      }
    };
    // A batch consumes at most one block of words.  While batch b runs, the pointer p_b it started from is
    // known here: the words down to p_b - 3 blocks are requested and those down to p_(b-1) - 3 blocks, at
    // or below p_b - 2 blocks, are in the ring -- batch b + 1 reads no further down than that.
    // With three blocks the words are staged two blocks below the pointer and none is left on its way: the
    // block written while batch b runs then takes the slot of the block three above it, which lies wholly
    // above the pointer batch b started from.
    constexpr int kBelow = (RB == 4 ? 3 : 2) * kBlockWords;
    stage_down_to(hi - kBelow, false);
    __syncthreads();  // barrier "start"
    int32_t ptr_before = hi;  // the pointer as it stood before the batch now running
    for (int32_t g0 = 0; g0 < G; g0 += kBatch) {
      stage_down_to(ptr_before - kBelow, RB == 4);
      __syncthreads();  // barrier of this batch: its symbols are in the stage, the pointer is published
      ptr_before = ptr_pub[(g0 / kBatch) & 1];  // (its own slot: the decoder publishes the next one a batch later)
      const bool tail = g0 >= g_tail;
      const int32_t cnt_groups = tail ? tail_groups : kBatch;
      const uint8_t *stage = sym_stage[(g0 / kBatch) & 1];
      const uint32_t done = (uint32_t)g0 * kLanes;
      const uint32_t room = (uint32_t)cnt_groups * kLanes;
      const uint32_t nsym = (len - done) < room ? (len - done) : room;
      if (out_aligned) {
        const uint32_t full = nsym / 16;
        if ((uint32_t)lane < full)
          *reinterpret_cast<uint4 *>(ubase + done + lane * 16) = *reinterpret_cast<const uint4 *>(&stage[lane * 16]);
        const uint32_t rest_at = full * 16 + (uint32_t)lane;
        if (rest_at < nsym) ubase[done + rest_at] = stage[rest_at];
      } else {
        for (uint32_t i = lane; i < nsym; i += 64) ubase[done + i] = stage[i];
      }
    }
    return;
  }

  // ---- the decoding wavefront
  // Lanes 0..31 decode.  Lanes 32..63 start as their copies and run the same instructions, so that no step
  // needs a lane mask; their ranks count all 32 decoding lanes, so their states go astray -- whatever they
  // read lies inside the tables, and what they store goes to a spare half of the stage.
  const bool coder = lane < kLanes;
  const int rl = lane & (kLanes - 1);
  const bool top_active = (uint32_t)rl < top_syms;
  const uint32_t x0 = a.states_in[unit * kLanes + rl];
  uint32_t xc = x0 >> kScaleBits;
  uint2 e = tab[x0 & (kScale - 1)];
  int32_t ptr = hi;
  __syncthreads();  // barrier "start": the first words are staged
  for (int32_t g0 = 0; g0 < G; g0 += kBatch) {
    const bool tail = g0 >= g_tail;
    const int32_t cnt_groups = tail ? tail_groups : kBatch;
    uint8_t *sb = &sym_stage[(g0 / kBatch) & 1][coder ? rl : kBatchSyms + rl];
    const uint32_t q0 = kRing - 1u - (uint32_t)(ptr - 1) % kRing;  // ring position of the top word (uniform)
    uint32_t ring_at = (uint32_t)kScale + q0;  // its entry in tab
    asm volatile("" : "+v"(ring_at));
    if (tail) {
      for (int32_t j = 0; j < cnt_groups; ++j)
        dec_chain_step<true>(xc, e, tab, ring_at, sb + kLanes * j, j != cnt_groups - 1 || top_active);
    } else {
#pragma unroll
      for (int j = 0; j < kBatch; ++j) dec_chain_step<false>(xc, e, tab, ring_at, sb + kLanes * j, true);
    }
    ptr -= (int32_t)((uint32_t)__builtin_amdgcn_readfirstlane(ring_at) - (uint32_t)kScale - q0);
    if (ptr < lo) {  // ran out of words: the stream is damaged
      bad = true;
      ptr = lo;
    }
    if (lane == 0) ptr_pub[(g0 / kBatch) & 1] = ptr;
    __syncthreads();  // barrier of this batch
  }
  // integrity: every word consumed, every lane back at the initial state: x >> 12 as carried, and the entry
  // in hand that of the initial state's slot with w4 = 0 (entries of different slots differ in .y, and
  // f * w4 > 0 otherwise)
  const uint2 e0 = tab[kLow & (kScale - 1)];
  const bool home = xc == (kLow >> kScaleBits) && e.x == e0.x && e.y == e0.y;
  if (ptr != lo || (coder && !home)) bad = true;
  if (bad) raise(a.status, PLC_ERR_CORRUPT);
}

// ---------------------------------------------------------------------------
// Decoder for streams coded as one unit with one table per bit depth
// ---------------------------------------------------------------------------
// The table changes from position to position, so when a word is staged the step that will consume it, and
// with it the table its slot will be looked up in, is not known.  There are at most PLC_MAX_BITS tables,
// though: the wavefront that stages a word looks its slot up in every one of them, and the ring holds one
// entry per word and table.  A step then has the one LDS round trip of the kernel above -- the ring entry of
// the next group's table for a lane that renormalises, that table's slot entry for a lane that does not, one
// read at an address chosen per lane.  For four rings and four tables to fit, an entry is 4 bytes and leaves
// the symbol out:
//   slot tables   per depth, 4 bytes per slot: f | (slot - cum) << 16                       (16 KB each)
//   rings         per depth, 4 bytes per word w: f | (f * (w >> 12) + slot - cum) << 16 with the slot
//                 w & 0xfff looked up in that depth's table (at most 4096 * 15 + 4095 = 2^16 - 1)
//   state         xh = x >> 12 without the bits the word supplies, as above: f * xh + (entry >> 16)
//   symbols       a step hands on where its entry was read from, as a 16-bit index of 4-byte words; the
//                 helper turns a batch of these into slots (a table word is its slot; a ring word names a
//                 word of the raw ring beside the rings, whose low 12 bits are the slot) and the slots into
//                 symbols through a 4 KB table per depth, while the next batch is decoded, and moves them out
//   step          multiply | add (each takes its half of the entry), compare, rank, select, shift | read:
//                 six dependent instructions and one round trip
// What a step costs is its dependent chain -- the round trip and six vector instructions at about eight cycles
// each, one more than the kernel above, whose entry needs no taking apart: 134 against 104 cycles a step with
// the barrier's share -- so the decoder's uniform operands are formed once per batch, and whatever else can
// be is left to the helper (handing on the slot itself, read by the decoder from the raw ring behind its
// entry, was tried: 2.4 against 2.1 ms on the Llama shape).  The helper stages the
// words, tells the decoder each batch's tables (16 tables in a word, two batches before they are needed; the
// depths come from global memory and are asked for a batch before that, their range looked at when they are
// used), turns the batch's entries' places into symbols and moves them out; it leaves a batch's barrier
// without waiting for its stores to be acknowledged.  With candidates a third wavefront reconstructs; it takes
// a batch's symbols from the helper, one barrier later than in the kernel above, and every wavefront joins one
// more barrier at the end.
//
// The same kernel with one table (MODE 1, and 2 with a chosen candidate per position) is the decoder that
// reconstructs for thousands of streams with k <= 4: the 4-byte entries and the symbols' table bring a workgroup
// to 39.2 KB of LDS, four to a compute unit instead of three with the 8-byte entries of the kernel above, and
// what counts there is how many streams are in flight, not one step's length (5120 streams, k = 4: 7.9 -> 7.0 ms).
constexpr uint32_t kDepthTableBytes = kScale * sizeof(uint32_t);
constexpr uint32_t kDepthSymBytes = kScale;
constexpr uint32_t kDepthRingSlots = kRingWords + kRingMirror;
constexpr uint32_t kDepthRingBytes = kDepthRingSlots * sizeof(uint32_t);
constexpr uint32_t kDepthRawBytes = kDepthRingSlots * sizeof(uint16_t);
static_assert(kDepthTableBytes % 16 == 0 && kDepthRingBytes % 16 == 0 && kDepthRawBytes % 16 == 0, "16-byte stores");
// dynamic LDS of the kernel: the slot tables, the rings, the raw ring, the symbol tables
inline size_t depths_lds_bytes(int n_tables) {
  return (size_t)n_tables * (kDepthTableBytes + kDepthRingBytes + kDepthSymBytes) + kDepthRawBytes;
}
constexpr int depths_threads(int rk) { return rk ? 192 : 128; }
static_assert(PLC_MAX_BITS * (kDepthTableBytes + kDepthRingBytes) / 4 <= 65536, "a word of the tables and rings in 16 bits");

// LDS of the kernel in 4-byte words.  tw is the first word of the next group's slot table, ring_at the word
// of that group's ring where the top word sits (both uniform; ring_at in a vector register), ring_step how far
// the ring that the step after this one reads lies behind this one's: ring_at for that step is formed here,
// behind the read, like everything else a step can do before its entry has arrived.  `at` is the word the
// entry in hand was read from; it is what a step hands on for its symbol.
template <bool MASKED>
__device__ __forceinline__ void dec_depth_step(uint32_t &xh, uint32_t &e, uint32_t &at, const uint32_t *lds_words,
                                               uint32_t &ring_at, uint16_t *code_slot, uint32_t tw,
                                               uint32_t ring_step, uint32_t slot_mask, bool on) {
  // f * (x >> 12) + slot - cum; product and sum kept apart so that each takes its half of the entry through
  // the instruction's own operand select instead of a mask and a shift in front of a fused multiply-add
  uint32_t fx = __umul24(e & 0xffffu, xh);
  asm volatile("" : "+v"(fx));
  const uint32_t xn = fx + (e >> 16);
  uint32_t m32 = (uint32_t)__builtin_amdgcn_uicmp(xn, kLow, 36 /* unsigned < */);
  bool need = xn < kLow;
  if (MASKED) {
    need = need && on;
    m32 = (uint32_t)__builtin_amdgcn_ballot_w64(need);
  }
  // ring entry of the rank-th word from the top, or slot-table entry of xn (tables start at multiples of 4096 words)
  uint32_t idx_ring = __builtin_amdgcn_mbcnt_lo(m32, ring_at);
  uint32_t idx_slot = (xn & slot_mask) | tw;  // (the mask in a register: and-or is one instruction then)
  asm volatile("" : "+v"(idx_ring), "+v"(idx_slot));  // both in registers: the choice is one select, not a branch
  const uint32_t at_next = need ? idx_ring : idx_slot;
  const uint32_t en = lds_words[at_next];
  __builtin_amdgcn_sched_barrier(0);  // what follows is issued in the shadow of the read
  ring_at += (uint32_t)__builtin_popcount(m32) + ring_step;
  asm volatile("" : "+v"(ring_at));
  const uint32_t next = need ? (xn << 4) : (xn >> kScaleBits);
  if (!MASKED || on) {
    *code_slot = (uint16_t)at;
    xh = next;
    e = en;
    at = at_next;
  }
  __builtin_amdgcn_sched_barrier(0);  // all of it before the entry is waited for
}

template <int RK, int MODE = 0>  // MODE 0: a table per depth; 1: one table; 2: one table and a chosen candidate
__global__ __launch_bounds__(depths_threads(RK)) void rans_decode_depths_kernel(const RansArgs a) {
  static_assert(MODE == 0 || RK > 0, "the one-table forms exist for the decoder that reconstructs");
  constexpr int RB = 4;  // ring blocks
  constexpr uint32_t kRing = kRingWords;
  constexpr int32_t kBelow = 3 * kBlockWords;  // how far below the pointer the words are staged
  const int n_tables = MODE ? 1 : a.n_tables;
  extern __shared__ __attribute__((aligned(16))) char depth_lds[];  // see depths_lds_bytes
  __shared__ __attribute__((aligned(16))) uint16_t code_stage[2][kBatchSyms];  // where the entries were read from
  __shared__ uint16_t code_spare[kBatchSyms];                                  // the same from lanes 32..63, never read
  __shared__ __attribute__((aligned(16))) uint8_t sym_stage[2][kBatchSyms];    // symbols, for the reconstruction
  uint32_t *const fc = reinterpret_cast<uint32_t *>(&code_stage[0][0]);        // frequencies while the tables are built
  static_assert(sizeof(code_stage) >= 256 * sizeof(uint32_t), "room for the frequencies");
  __shared__ uint32_t tables_of_batch[4];  // batch b mod 4: the tables of groups 16 b + 1 .. 16 b + 16, two bits each
  __shared__ uint32_t first_table;
  __shared__ int32_t ptr_pub[2];  // the word pointer after batch b, in slot b mod 2
  __shared__ uint32_t tables_ok;
  constexpr int kThreads = depths_threads(RK);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const bool helper = wave == 1;
  const int64_t stream = blockIdx.x / a.wgs_per_stream;
  const int64_t chunk = blockIdx.x - stream * a.wgs_per_stream;
  const uint32_t ring_off = (uint32_t)n_tables * kDepthTableBytes;
  const uint32_t raw_off = ring_off + (uint32_t)n_tables * kDepthRingBytes;
  const uint32_t symtab_off = raw_off + kDepthRawBytes;
  bool bad = false;

  // slot and symbol tables, one depth after the other; an all-zero table (a depth the stream does not use)
  // stays zero
  if (threadIdx.x == 0) tables_ok = 1u;
  __syncthreads();
  uint32_t used = 0;  // uniform: bit t set when table t is one
  for (int t = 0; t < n_tables; ++t) {
    uint32_t f[4], cum;
    const uint32_t total = load_freq4(a.freq + (stream * n_tables + t) * 256, lane, f, &cum);
    if (total != kScale && (MODE || total != 0) && threadIdx.x == 0) tables_ok = 0u;
    if (wave == 0) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        fc[lane * 4 + r] = f[r] | (cum << 16);
        cum += f[r];
      }
    }
    __syncthreads();
    uint32_t *tt = reinterpret_cast<uint32_t *>(depth_lds + (size_t)t * kDepthTableBytes);
    uint8_t *ts = reinterpret_cast<uint8_t *>(depth_lds + symtab_off + (size_t)t * kDepthSymBytes);
    if (total == kScale) {
      used |= 1u << t;
      for (int sy = 0; sy < 256; ++sy) {
        const uint32_t v = fc[sy];
        const uint32_t fs = v & 0xffffu, cs = v >> 16;
        for (uint32_t o = threadIdx.x; o < fs; o += kThreads) {
          tt[cs + o] = fs | (o << 16);
          ts[cs + o] = (uint8_t)sy;
        }
      }
    } else {
      for (uint32_t o = threadIdx.x; o < (uint32_t)kScale; o += kThreads) tt[o] = 0u, ts[o] = 0;
    }
    __syncthreads();
  }
  if (!tables_ok) {  // not a table: nothing can be decoded (uniform: every wavefront leaves)
    if (threadIdx.x == 0) raise(a.status, PLC_ERR_CORRUPT);
    return;
  }

  const int64_t unit = stream * a.units_per_stream + chunk;
  const int64_t begin = chunk * a.unit_syms;
  const int64_t rest = a.syms_per_stream - begin;
  const uint32_t len = (uint32_t)(rest < a.unit_syms ? rest : a.unit_syms);
  const int32_t G = (int32_t)((len + kLanes - 1) / kLanes);
  const uint32_t top_syms = len - (uint32_t)(G - 1) * kLanes;

  const uint64_t off = a.word_off[unit];
  const uint32_t n = a.n_words_in[unit];
  if (off > a.words_len || (uint64_t)n > a.words_len - off) {  // uniform: every wavefront leaves
    if (threadIdx.x == 0) raise(a.status, PLC_ERR_CORRUPT);
    return;
  }
  const uint16_t *first_word = a.words_in + off;
  const int32_t lo = (int32_t)((reinterpret_cast<uintptr_t>(first_word) & (uintptr_t)(kBlockWords * 2 - 1)) >> 1);
  const uint16_t *aligned_base = first_word - lo;
  const int32_t hi = lo + (int32_t)n;

  int32_t tail_groups = G % kBatch;
  if (tail_groups == 0 && top_syms < kLanes) tail_groups = kBatch;
  const int32_t g_tail = G - tail_groups;

  if constexpr (RK > 0) {  // the wavefront that reconstructs, one barrier behind the decoder's batch
    if (wave == 2) {
      reconstruct_batches<RK, MODE != 1, MODE == 0, kRecDepthBase, 1, kBatchSyms>(a, stream, len, G, sym_stage, lane);
      return;
    }
  }

  if (helper) {
    bool bad_depth = false;
    uint8_t *ubase = a.sym_out + stream * a.syms_per_stream + begin;
    const bool out_aligned = (reinterpret_cast<uintptr_t>(ubase) & 7u) == 0;
    auto block_load = [&](int32_t blk, uint4 &v) -> bool {
      const int32_t first = blk * kBlockWords + lane * 8;
      const bool take = blk >= 0 && hi > lo && first + 8 > lo && first < hi;
      if (take) v = *reinterpret_cast<const uint4 *>(aligned_base + first);
      return take;
    };
    // word i goes to ring position (~i) mod 2048: the lane's eight words, last one first
    auto block_store = [&](int32_t blk, bool take, const uint4 &v) {
      if (take) {
        // word i sits at ring position kRing - 1 - i mod kRing; this is the lane's last word's
        const uint32_t pos = (uint32_t)((RB - 1 - blk % RB) * kBlockWords + (kBlockWords - 8 - lane * 8));
        const uint32_t w[8] = {v.w >> 16, v.w & 0xffffu, v.z >> 16, v.z & 0xffffu,
                               v.y >> 16, v.y & 0xffffu, v.x >> 16, v.x & 0xffffu};
        const uint4 rw = make_uint4(w[0] | (w[1] << 16), w[2] | (w[3] << 16), w[4] | (w[5] << 16), w[6] | (w[7] << 16));
        char *raw = depth_lds + raw_off;
        *reinterpret_cast<uint4 *>(raw + pos * 2) = rw;
        if (pos < (uint32_t)kRingMirror) *reinterpret_cast<uint4 *>(raw + (kRing + pos) * 2) = rw;
        for (int t = 0; t < n_tables; ++t) {  // uniform
          if (!((used >> t) & 1u)) continue;    // a depth without a table is never looked up
          const uint32_t *tt = reinterpret_cast<const uint32_t *>(depth_lds + (size_t)t * kDepthTableBytes);
          uint32_t en[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const uint32_t s = tt[w[i] & (kScale - 1)];
            en[i] = s + (__umul24(s & 0xffffu, w[i] >> kScaleBits) << 16);
          }
          uint32_t *ring = reinterpret_cast<uint32_t *>(depth_lds + ring_off + (size_t)t * kDepthRingBytes);
          const uint4 r0 = make_uint4(en[0], en[1], en[2], en[3]), r1 = make_uint4(en[4], en[5], en[6], en[7]);
          *reinterpret_cast<uint4 *>(&ring[pos]) = r0;
          *reinterpret_cast<uint4 *>(&ring[pos + 4]) = r1;
          if (pos < (uint32_t)kRingMirror) {
            *reinterpret_cast<uint4 *>(&ring[kRing + pos]) = r0;
            *reinterpret_cast<uint4 *>(&ring[kRing + pos + 4]) = r1;
          }
        }
      }
    };
    // as in the kernel above: the newest block stays on its way for a batch
    int32_t lowest = ((hi - 1) >> 9) + 1;  // lowest block already requested (none yet)
    uint4 ahead_v;
    int32_t ahead_blk = 0;
    bool ahead = false, ahead_take = false;
    auto stage_down_to = [&](int32_t down_to, bool leave_one) {
      if (ahead) {  // uniform
        block_store(ahead_blk, ahead_take, ahead_v);
        ahead = false;
      }
      const int32_t last = down_to > 0 ? down_to >> 9 : 0;
      while (lowest > last) {
        const int32_t blk = lowest - 1;
        lowest = blk;
        if (leave_one && blk == last) {
          ahead_take = block_load(blk, ahead_v);
          ahead_blk = blk;
          ahead = true;
        } else {
          uint4 v;
          const bool take = block_load(blk, v);
          block_store(blk, take, v);
        }
      }
    };
    // Tables of groups g0 + 1 .. g0 + 16, the ones the 16 steps of the batch at g0 look up (past the last
    // group: the first table, whose entry is never used).  A depth is asked for here and looked at a batch
    // later (in range or not included), when it is packed with the 15 others for the decoder.
    static_assert(PLC_MAX_BITS <= 4 && kBatch == 16, "two bits per table, 16 tables in a word");
    const uint32_t spp = MODE ? 1u : (uint32_t)a.syms_per_pos;  // (one table: no depths, nothing below is reached)
    const uint8_t *depth_row =
        MODE ? nullptr
             : a.bits + (int64_t)((uint32_t)stream / (uint32_t)a.streams_per_session) * ((uint32_t)a.syms_per_stream / spp);
    auto fetch_depths = [&](int32_t g0) -> uint32_t {
      const int32_t g = g0 + 1 + (lane & (kBatch - 1));
      return g < G ? depth_row[(uint32_t)(begin + (int64_t)g * kLanes) / spp] : 1u;
    };
    auto pack_tables = [&](uint32_t depth) -> uint32_t {  // lanes 0..15 hold a depth each
      if (depth < 1u || depth > (uint32_t)a.n_tables) {
        bad_depth = true;
        depth = 1u;
      }
      uint32_t v = (depth - 1u) << (2 * (lane & (kBatch - 1)));
#pragma unroll
      for (int off = 1; off < kBatch; off <<= 1) v |= __shfl_xor(v, off, 64);
      return (uint32_t)__builtin_amdgcn_readfirstlane(v);
    };
    stage_down_to(hi - kBelow, false);
    uint32_t t_first = 0, tables_cur = 0, tables_next = 0, depth_ahead = 1;
    if constexpr (MODE == 0) {
      t_first = group_table(a, stream, begin, 0, 1u, &bad_depth);  // table of the coming batch's first group
      tables_cur = pack_tables(fetch_depths(0)), tables_next = pack_tables(fetch_depths(kBatch));
      if (lane == 0) {
        first_table = t_first;
        tables_of_batch[0] = tables_cur;
        tables_of_batch[1] = tables_next;
      }
      depth_ahead = fetch_depths(2 * kBatch);
    }
    __syncthreads();  // barrier "start"
    int32_t ptr_before = hi;
    for (int32_t g0 = 0; g0 < G; g0 += kBatch) {
      stage_down_to(ptr_before - kBelow, true);
      uint32_t tables_after = 0;
      if constexpr (MODE == 0) {
        tables_after = pack_tables(depth_ahead);
        if (lane == 0) tables_of_batch[((g0 / kBatch) + 2) & 3] = tables_after;
        depth_ahead = fetch_depths(g0 + 3 * kBatch);
      }
      lds_barrier();  // barrier of this batch
      // (The pointer has a slot per batch parity: this wavefront may still be waiting for its loads from global
      // memory, which the barrier above does not wait for, when the decoder publishes the pointer after the next
      // batch; read from a single slot it then stages a block too early, over words whose places are yet to be
      // turned into symbols.)
      ptr_before = ptr_pub[(g0 / kBatch) & 1];
      // the table of the group this lane's eight entries of the batch belong to: the one the step before
      // looked up (for the batch's first group: the last of the batch before)
      const uint32_t t_mine = (lane >> 2) == 0 ? t_first : (tables_cur >> (2 * ((lane >> 2) - 1))) & 3u;
      t_first = tables_cur >> 30;
      tables_cur = tables_next;
      tables_next = tables_after;
      const bool tail = g0 >= g_tail;
      const int32_t cnt_groups = tail ? tail_groups : kBatch;
      const int buf = (g0 / kBatch) & 1;
      const uint32_t done = (uint32_t)g0 * kLanes;
      const uint32_t room = (uint32_t)cnt_groups * kLanes;
      const uint32_t nsym = (len - done) < room ? (len - done) : room;
      // where each entry was read from -> slot -> symbol, eight per lane
      const uint4 cv = *reinterpret_cast<const uint4 *>(&code_stage[buf][lane * 8]);
      const uint8_t *ts = reinterpret_cast<const uint8_t *>(depth_lds + symtab_off + (size_t)t_mine * kDepthSymBytes);
      const uint16_t *raw = reinterpret_cast<const uint16_t *>(depth_lds + raw_off);
      const uint32_t ring_word0 = ring_off / 4 + t_mine * kDepthRingSlots;  // of this group's ring
      const uint32_t c[8] = {cv.x & 0xffffu, cv.x >> 16, cv.y & 0xffffu, cv.y >> 16,
                             cv.z & 0xffffu, cv.z >> 16, cv.w & 0xffffu, cv.w >> 16};
      // (every lane reads the raw ring, needed or not, and all eight reads are on their way before the first
      // is used: two LDS round trips for the batch, not sixteen)
      uint32_t word[8], sy[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        uint32_t p = c[i] - ring_word0;  // not a ring word, or a lane past the end of the stream: keep inside
        p = p < kDepthRingSlots ? p : 0u;
        word[i] = raw[p];
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint32_t slot_i = c[i] >= ring_off / 4 ? word[i] : c[i];
        sy[i] = ts[slot_i & (kScale - 1)];
      }
      const uint2 sv = make_uint2(sy[0] | (sy[1] << 8) | (sy[2] << 16) | (sy[3] << 24),
                                  sy[4] | (sy[5] << 8) | (sy[6] << 16) | (sy[7] << 24));
      if constexpr (RK > 0) *reinterpret_cast<uint2 *>(&sym_stage[buf][lane * 8]) = sv;
      const uint32_t mine = (uint32_t)lane * 8;
      if (out_aligned && mine + 8 <= nsym) {
        *reinterpret_cast<uint2 *>(ubase + done + mine) = sv;
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i)
          if (mine + i < nsym) ubase[done + mine + i] = (uint8_t)sy[i];
      }
      // (the raw ring is read above as 16-bit words and written by the staging below as 16-byte vectors: the
      // accesses are kept in this order whatever the compiler makes of their types)
      asm volatile("" ::: "memory");
    }
    if constexpr (RK > 0) lds_barrier();  // the last batch's symbols are in the stage
    if (bad_depth) raise(a.status, PLC_ERR_INVALID);
    return;
  }

  // ---- the decoding wavefront (lanes 32..63 ride along, as in the kernel above)
  const bool coder = lane < kLanes;
  const int rl = lane & (kLanes - 1);
  const bool top_active = (uint32_t)rl < top_syms;
  const uint32_t x0 = a.states_in[unit * kLanes + rl];
  int32_t ptr = hi;
  __syncthreads();  // barrier "start": the first words are staged, the first tables known
  const uint32_t *lds_words = reinterpret_cast<const uint32_t *>(depth_lds);
  uint32_t slot_mask = kScale - 1;
  asm volatile("" : "+v"(slot_mask));
  uint32_t xh = x0 >> kScaleBits;
  uint32_t at = (MODE ? 0u : first_table * kScale) + (x0 & (kScale - 1));
  uint32_t e = lds_words[at];
  uint32_t tables = MODE ? 0u : (uint32_t)__builtin_amdgcn_readfirstlane(tables_of_batch[0]);
  const uint32_t ring0 = ring_off / 4;
  for (int32_t g0 = 0; g0 < G; g0 += kBatch) {
    const bool tail = g0 >= g_tail;
    const int32_t cnt_groups = tail ? tail_groups : kBatch;
    // (the next batch's tables: asked for now, used after the barrier)
    const uint32_t tables_coming = MODE ? 0u : tables_of_batch[((g0 / kBatch) + 1) & 3];
    uint16_t *sb = coder ? &code_stage[(g0 / kBatch) & 1][rl] : &code_spare[rl];
    const uint32_t q0 = kRing - 1u - (uint32_t)(ptr - 1) % kRing;  // ring position of the top word (uniform)
    uint32_t ring_at = ring0 + (tables & 3u) * kDepthRingSlots + q0;
    asm volatile("" : "+v"(ring_at));
    if (tail) {
      for (int32_t j = 0; j < cnt_groups; ++j) {
        const uint32_t t = (tables >> (2 * j)) & 3u, t_after = j + 1 < kBatch ? (tables >> (2 * j + 2)) & 3u : 0u;
        dec_depth_step<true>(xh, e, at, lds_words, ring_at, sb + kLanes * j, t * kScale,
                             (t_after - t) * kDepthRingSlots, slot_mask, j != cnt_groups - 1 || top_active);
      }
    } else {
      // every step's two uniform operands, formed before the first step (in scalar registers from here on)
      uint32_t tw[kBatch], rs[kBatch];
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        const uint32_t t = (tables >> (2 * j)) & 3u, t_after = j + 1 < kBatch ? (tables >> (2 * j + 2)) & 3u : 0u;
        tw[j] = t * kScale;
        rs[j] = (t_after - t) * kDepthRingSlots;
        asm volatile("" : "+s"(tw[j]), "+s"(rs[j]));
      }
#pragma unroll
      for (int j = 0; j < kBatch; ++j)
        dec_depth_step<false>(xh, e, at, lds_words, ring_at, sb + kLanes * j, tw[j], rs[j], slot_mask, true);
    }
    // (The entry in hand is handed on with the next batch's first step, and where it was read from is looked at
    // a barrier after that.  If it is a ring word it is still there then: the block staged in between goes
    // where a block above the pointer of a batch ago was, and the word is below that pointer.)
    // the ring position is now the first ring's (table 0 stands in past the batch's last group) plus the words taken
    ptr -= (int32_t)((uint32_t)__builtin_amdgcn_readfirstlane(ring_at) - ring0 - q0);
    if (ptr < lo) {
      bad = true;
      ptr = lo;
    }
    if (lane == 0) ptr_pub[(g0 / kBatch) & 1] = ptr;
    __syncthreads();  // barrier of this batch
    tables = MODE ? 0u : (uint32_t)__builtin_amdgcn_readfirstlane(tables_coming);
  }
  if constexpr (RK > 0) __syncthreads();  // the helper's last batch of symbols, for the reconstruction
  // integrity: every word consumed, every lane back at the initial state: x >> 12 as carried, and slot 0, which
  // the place of the entry in hand tells (the helper stages nothing after the last batch's barrier)
  uint32_t slot;
  if (at >= ring0) {
    const uint32_t p = (at - ring0) % kDepthRingSlots;
    slot = reinterpret_cast<const uint16_t *>(depth_lds + raw_off)[p] & (kScale - 1);
  } else {
    slot = at & (kScale - 1);
  }
  const bool home = xh == (kLow >> kScaleBits) && slot == 0u;
  if (ptr != lo || (coder && !home)) bad = true;
  if (bad) raise(a.status, PLC_ERR_CORRUPT);
}

int check_common(int64_t n_streams, int64_t syms_per_stream, int32_t chunk_syms, RansArgs *a, int *waves) {
  if (n_streams < 1 || syms_per_stream < 1) return PLC_ERR_INVALID;
  if (syms_per_stream >= (1ll << 31) - 1024) return PLC_ERR_INVALID;
  if (chunk_syms < 0 || chunk_syms % kLanes) return PLC_ERR_INVALID;
  a->units_per_stream = plc_units_per_stream(syms_per_stream, chunk_syms);
  a->unit_syms = chunk_syms > 0 ? chunk_syms : syms_per_stream;
  a->n_units = n_streams * a->units_per_stream;
  a->syms_per_stream = syms_per_stream;
  int w = 1;
  while (w < kMaxWaves && 2 * w <= a->units_per_stream) w *= 2;
  *waves = w;
  const int64_t wgs = (a->units_per_stream + w - 1) / w;
  if (wgs >= (1ll << 31) || n_streams * wgs >= (1ll << 31)) return PLC_ERR_INVALID;
  a->wgs_per_stream = (uint32_t)wgs;
  return PLC_OK;
}

template <template <int> class Launcher>
void dispatch_waves(int waves, const RansArgs &a, unsigned grid, hipStream_t st) {
  switch (waves) {
    case 1: Launcher<1>::run(a, grid, st); break;
    case 2: Launcher<2>::run(a, grid, st); break;
    case 4: Launcher<4>::run(a, grid, st); break;
    default: Launcher<8>::run(a, grid, st); break;
  }
}

template <int W>
struct LaunchEncode {
  static void run(const RansArgs &a, unsigned grid, hipStream_t st) {
    if (a.bits) {
      hipLaunchKernelGGL((rans_encode_kernel<W, true>), dim3(grid), dim3(W * 64), 0, st, a);
    } else {
      hipLaunchKernelGGL((rans_encode_kernel<W, false>), dim3(grid), dim3(W * 64), 0, st, a);
    }
  }
};
template <int W>
struct LaunchDecode {
  static void run(const RansArgs &a, unsigned grid, hipStream_t st) {
    // One unit per stream and few enough units (kChainMaxUnits): time is the length of one unit's chain,
    // so take the variant with the shortest step.  With more units its 60 KB of LDS per workgroup would
    // cost more in occupancy than the shorter step gains.
    if (a.bits && W == 1 && a.n_units <= kDepthsMaxUnits) {
      const size_t lds = depths_lds_bytes(a.n_tables);
      (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&rans_decode_depths_kernel<0>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      hipLaunchKernelGGL(rans_decode_depths_kernel<0>, dim3(grid), dim3(depths_threads(0)), lds, st, a);
    } else if (a.bits) {
      // (the split tables here too: 5 KB per depth instead of 16 lets three times the wavefronts in)
      const size_t lds = (size_t)a.n_tables * kCompactTable * sizeof(uint32_t);
      (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&rans_decode_kernel<W, true, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      hipLaunchKernelGGL((rans_decode_kernel<W, true, true>), dim3(grid), dim3(W * 64), lds, st, a);
    } else if (W == 1 && a.n_units <= kChainMaxUnits) {
      hipLaunchKernelGGL((rans_decode_chain_kernel<0, false>), dim3(grid), dim3(128), 0, st, a);
    } else {
      // Many units: LDS decides how many wavefronts fit a compute unit, and the split table lets more in
      // (twice as many where every one-wavefront workgroup has a table of its own).
      hipLaunchKernelGGL((rans_decode_kernel<W, false, true>), dim3(grid), dim3(W * 64), 0, st, a);
    }
  }
};

}  // namespace
}  // namespace plc

using namespace plc;

extern "C" int64_t plc_units_per_stream(int64_t syms_per_stream, int32_t chunk_syms) {
  if (chunk_syms <= 0) return 1;
  return (syms_per_stream + chunk_syms - 1) / chunk_syms;
}

namespace plc {
namespace {

// Arguments of the calls with one table per bit depth.
int check_depths(int64_t syms_per_stream, int32_t chunk_syms, int32_t syms_per_pos, int32_t streams_per_session,
                 const uint8_t *bits, int32_t n_tables, RansArgs *a) {
  if (!bits || n_tables < 1 || n_tables > PLC_MAX_BITS || streams_per_session < 1) return PLC_ERR_INVALID;
  if (syms_per_pos < kLanes || syms_per_pos % kLanes || syms_per_stream % syms_per_pos) return PLC_ERR_INVALID;
  (void)chunk_syms;  // a multiple of 32 already: groups never straddle positions
  a->bits = bits;
  a->syms_per_pos = syms_per_pos;
  a->streams_per_session = streams_per_session;
  a->n_tables = n_tables;
  return PLC_OK;
}

int encode_impl(const uint8_t *symbols, int64_t n_streams, int64_t syms_per_stream, int32_t chunk_syms,
                const uint16_t *freq, uint32_t *states, uint16_t *words, const uint64_t *word_off,
                uint64_t word_cap_per_unit, uint32_t *n_words, uint32_t *status, void *stream, RansArgs a) {
  int waves = 1;
  int rc = check_common(n_streams, syms_per_stream, chunk_syms, &a, &waves);
  if (rc) return rc;
  if (!symbols || !freq || !states || !word_off || !n_words || !status) return PLC_ERR_INVALID;
  if (word_cap_per_unit > 0 && !words) return PLC_ERR_INVALID;
  if (reinterpret_cast<uintptr_t>(freq) % 8 || reinterpret_cast<uintptr_t>(words) % 2) return PLC_ERR_INVALID;
  a.sym_in = symbols;
  a.freq = freq;
  a.states_out = states;
  a.words_out = words;
  a.word_off = word_off;
  a.word_cap = word_cap_per_unit;
  a.n_words_out = n_words;
  a.status = status;
  hipStream_t st = static_cast<hipStream_t>(stream);
  {
    TraceScope trace(PLC_TRACE_RANS_ENCODE, st);
    if (a.units_per_stream == 1 && a.n_units <= kPipeMaxUnits) {
      // few units (kPipeMaxUnits): the chain of one unit is the time, so give each unit three wavefronts
      // (with more units, three wavefronts per unit cost more in occupancy than the shorter chain gains)
      if (a.bits) {
        hipLaunchKernelGGL(rans_encode_pipe_kernel<true>, dim3((unsigned)a.n_units), dim3(192), 0, st, a);
      } else {
        hipLaunchKernelGGL(rans_encode_pipe_kernel<false>, dim3((unsigned)a.n_units), dim3(192), 0, st, a);
      }
    } else if (a.bits) {
      dispatch_waves<LaunchEncode>(waves, a, (unsigned)(n_streams * a.wgs_per_stream), st);
    } else if (a.units_per_stream == 1) {
      // many whole streams: two streams per wavefront, one wavefront per workgroup
      const int64_t pairs = (a.n_units + 1) / 2;
      if (pairs > 8 * kComputeUnits && pairs <= 11 * kComputeUnits) {  // all resident at once with the smaller stages
        hipLaunchKernelGGL((rans_encode_pair_kernel<1, true, 2>), dim3((unsigned)pairs), dim3(64), 0, st, a);
      } else {
        hipLaunchKernelGGL((rans_encode_pair_kernel<1, true, 4>), dim3((unsigned)pairs), dim3(64), 0, st, a);
      }
    } else {
      // chunks: two chunks of full length per wavefront; an odd one and a shorter last chunk take a wavefront each
      const int64_t n_full = a.syms_per_stream / a.unit_syms;
      const int64_t slots = n_full / 2 + (n_full & 1) + (n_full < a.units_per_stream ? 1 : 0);
      int w = 1;
      while (w < kPairMaxWaves && 2 * w <= slots) w *= 2;
      a.pair_wgs_per_stream = (uint32_t)((slots + w - 1) / w);
      const unsigned grid = (unsigned)(n_streams * a.pair_wgs_per_stream);  // at most the grid checked above
      switch (w) {
        case 1: hipLaunchKernelGGL((rans_encode_pair_kernel<1, false>), dim3(grid), dim3(64), 0, st, a); break;
        case 2: hipLaunchKernelGGL((rans_encode_pair_kernel<2, false>), dim3(grid), dim3(128), 0, st, a); break;
        default: hipLaunchKernelGGL((rans_encode_pair_kernel<4, false>), dim3(grid), dim3(256), 0, st, a); break;
      }
    }
  }
  return launch_status();
}

int decode_impl(const uint16_t *freq, const uint32_t *states, const uint16_t *words, uint64_t words_len,
                const uint64_t *word_off, const uint32_t *n_words, int64_t n_streams, int64_t syms_per_stream,
                int32_t chunk_syms, uint8_t *symbols, uint32_t *status, void *stream, RansArgs a) {
  int waves = 1;
  int rc = check_common(n_streams, syms_per_stream, chunk_syms, &a, &waves);
  if (rc) return rc;
  if (!symbols || !freq || !states || !word_off || !n_words || !status) return PLC_ERR_INVALID;
  if (words_len > 0 && !words) return PLC_ERR_INVALID;
  if (reinterpret_cast<uintptr_t>(freq) % 8 || reinterpret_cast<uintptr_t>(words) % 2) return PLC_ERR_INVALID;
  a.sym_out = symbols;
  a.freq = freq;
  a.states_in = states;
  a.words_in = words;
  a.words_len = words_len;
  a.word_off = word_off;
  a.n_words_in = n_words;
  a.status = status;
  hipStream_t st = static_cast<hipStream_t>(stream);
  {
    TraceScope trace(PLC_TRACE_RANS_DECODE, st);
    dispatch_waves<LaunchDecode>(waves, a, (unsigned)(n_streams * a.wgs_per_stream), st);
  }
  return launch_status();
}

}  // namespace

bool decode_fused_supported(int64_t n_streams, int64_t syms_per_stream, int k, bool cond, bool per_depth) {
  // Candidates that fit the registers of one wavefront kRecDepth batches deep, and whole chunks.  As to
  // the number of streams: two or three workgroups per compute unit run at a time, and a round takes its
  // chain's time or the HBM time of its reconstruction, whichever is longer.  With the weighted mean the two
  // are of a size, so the kernel beats the many-unit decoder followed by the reconstruction kernel however
  // many rounds there are (5120 streams: 7.9 against 10.9 ms; 16,384 streams with k = 8: 31 against 42 ms).
  // The token-conditional reconstruction moves a quarter of the bytes, so there is little to hide: with
  // k <= 4, where three workgroups share a compute unit, the kernel still wins (5120 streams: 7.0 against
  // 7.9 ms); with more candidates (two workgroups) the many-unit decoder's shorter total wins from some eight
  // rounds on (16,384 streams, k = 8: 28.4 against 22.5 ms): 2048 streams at most.  With one table per depth a
  // round is 256 workgroups, and the bound of that decoder applies.
  const int64_t most = per_depth ? kDepthsMaxUnits : (cond && k > 4) ? 2048 : INT64_MAX;
  return n_streams >= 1 && n_streams <= most && k >= 1 && k <= 8 && syms_per_stream >= kChunk &&
         syms_per_stream % kChunk == 0;
}

int rans_decode_fused(const uint16_t *freq, const uint32_t *states, const uint16_t *words, uint64_t words_len,
                      const uint64_t *word_off, const uint32_t *n_words, int64_t n_streams,
                      int64_t syms_per_stream, int32_t n_tables, uint8_t *symbols, const ReconView &recon,
                      uint32_t *status, hipStream_t st, bool launch) {
  RansArgs a = {};
  int waves = 1;
  int rc = check_common(n_streams, syms_per_stream, 0, &a, &waves);
  if (rc) return rc;
  if (!decode_fused_supported(n_streams, syms_per_stream, recon.k, recon.chosen != nullptr, recon.bits != nullptr))
    return PLC_ERR_INVALID;
  if (!symbols || !freq || !states || !word_off || !n_words || !status) return PLC_ERR_INVALID;
  if (words_len > 0 && !words) return PLC_ERR_INVALID;
  if (reinterpret_cast<uintptr_t>(freq) % 8 || reinterpret_cast<uintptr_t>(words) % 2) return PLC_ERR_INVALID;
  if ((int64_t)recon.L * recon.H < 1 || n_streams % ((int64_t)recon.L * recon.H)) return PLC_ERR_INVALID;
  if (syms_per_stream != 2ll * recon.n * recon.d8 * kChunk) return PLC_ERR_INVALID;
  if (recon.bits) {  // one table per bit depth: a position is the 2 * d symbols of its K and V rows
    if (!recon.chosen || !(recon.range > 0.0f)) return PLC_ERR_INVALID;
    rc = check_depths(syms_per_stream, 0, 2 * recon.d8 * kChunk, recon.L * recon.H, recon.bits, n_tables, &a);
    if (rc) return rc;
  }
  if (!launch) return PLC_OK;
  a.sym_out = symbols;
  a.freq = freq;
  a.states_in = states;
  a.words_in = words;
  a.words_len = words_len;
  a.word_off = word_off;
  a.n_words_in = n_words;
  a.status = status;
  a.recon = recon;
  {
    TraceScope trace(PLC_TRACE_RANS_DECODE, st);
    const dim3 grid((unsigned)n_streams), block(192);
    const size_t lds = depths_lds_bytes(a.n_tables);
    switch (recon.k) {
#define PLC_CASE(K)                                                                              \
  case K:                                                                                        \
    if (recon.bits) {                                                                            \
      (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&rans_decode_depths_kernel<K>),   \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);           \
      hipLaunchKernelGGL(rans_decode_depths_kernel<K>, grid, dim3(depths_threads(K)), lds, st, a); \
    } else if (K <= kCompactMaxK && n_streams > kDenseStreams) {                                 \
      const size_t lds1 = depths_lds_bytes(1);                                                \
      if (recon.chosen) {                                                                        \
        hipLaunchKernelGGL((rans_decode_depths_kernel<(K <= kCompactMaxK ? K : 1), 2>), grid, block, lds1, st, a); \
      } else {                                                                                   \
        hipLaunchKernelGGL((rans_decode_depths_kernel<(K <= kCompactMaxK ? K : 1), 1>), grid, block, lds1, st, a); \
      }                                                                                          \
    } else if (recon.chosen) {                                                                   \
      hipLaunchKernelGGL((rans_decode_chain_kernel<K, true>), grid, block, 0, st, a);            \
    } else if (K <= kDenseMaxK && n_streams > kDenseStreams) {                                   \
      hipLaunchKernelGGL((rans_decode_chain_kernel<(K <= kDenseMaxK ? K : 1), false, 3>), grid, block, 0, st, a); \
    } else {                                                                                     \
      hipLaunchKernelGGL((rans_decode_chain_kernel<K, false>), grid, block, 0, st, a);           \
    }                                                                                            \
    break;
      PLC_CASE(1) PLC_CASE(2) PLC_CASE(3) PLC_CASE(4) PLC_CASE(5) PLC_CASE(6) PLC_CASE(7) PLC_CASE(8)
#undef PLC_CASE
      default: return PLC_ERR_INVALID;
    }
  }
  return launch_status();
}

}  // namespace plc

extern "C" int plc_rans_encode(const uint8_t *symbols, int64_t n_streams, int64_t syms_per_stream,
                               int32_t chunk_syms, const uint16_t *freq, uint32_t *states, uint16_t *words,
                               const uint64_t *word_off, uint64_t word_cap_per_unit, uint32_t *n_words,
                               uint32_t *status, void *stream) {
  return encode_impl(symbols, n_streams, syms_per_stream, chunk_syms, freq, states, words, word_off,
                     word_cap_per_unit, n_words, status, stream, RansArgs{});
}

extern "C" int plc_rans_decode(const uint16_t *freq, const uint32_t *states, const uint16_t *words,
                               uint64_t words_len, const uint64_t *word_off, const uint32_t *n_words,
                               int64_t n_streams, int64_t syms_per_stream, int32_t chunk_syms, uint8_t *symbols,
                               uint32_t *status, void *stream) {
  return decode_impl(freq, states, words, words_len, word_off, n_words, n_streams, syms_per_stream, chunk_syms,
                     symbols, status, stream, RansArgs{});
}

extern "C" int plc_rans_encode_bucketed(const uint8_t *symbols, int64_t n_streams, int64_t syms_per_stream,
                                        int32_t chunk_syms, int32_t syms_per_pos, int32_t streams_per_session,
                                        const uint8_t *bits, int32_t n_tables, const uint16_t *freq,
                                        uint32_t *states, uint16_t *words, const uint64_t *word_off,
                                        uint64_t word_cap_per_unit, uint32_t *n_words, uint32_t *status,
                                        void *stream) {
  RansArgs a = {};
  const int rc = check_depths(syms_per_stream, chunk_syms, syms_per_pos, streams_per_session, bits, n_tables, &a);
  if (rc) return rc;
  return encode_impl(symbols, n_streams, syms_per_stream, chunk_syms, freq, states, words, word_off,
                     word_cap_per_unit, n_words, status, stream, a);
}

extern "C" int plc_rans_decode_bucketed(const uint16_t *freq, const uint32_t *states, const uint16_t *words,
                                        uint64_t words_len, const uint64_t *word_off, const uint32_t *n_words,
                                        int64_t n_streams, int64_t syms_per_stream, int32_t chunk_syms,
                                        int32_t syms_per_pos, int32_t streams_per_session, const uint8_t *bits,
                                        int32_t n_tables, uint8_t *symbols, uint32_t *status, void *stream) {
  RansArgs a = {};
  const int rc = check_depths(syms_per_stream, chunk_syms, syms_per_pos, streams_per_session, bits, n_tables, &a);
  if (rc) return rc;
  return decode_impl(freq, states, words, words_len, word_off, n_words, n_streams, syms_per_stream, chunk_syms,
                     symbols, status, stream, a);
}
