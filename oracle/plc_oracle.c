/*
 * plc_oracle.c -- CPU oracle for predictive delta coding of a KV cache.
 *
 * TEST INFRASTRUCTURE ONLY (see plc_oracle.h).  Plain scalar C, one symbol at
 * a time, in the order the format is defined in; nothing here is blocked,
 * fused or reordered.  Build with -ffp-contract=off so that the compiler never
 * fuses a multiply and an add the text below keeps apart.
 */
#include "plc_oracle.h"

#include <math.h>
#include <stddef.h>
#include <string.h>

#define RANS_LANES 32
#define RANS_SCALE_BITS 12
#define RANS_SCALE (1u << RANS_SCALE_BITS) /* frequencies sum to this      */
#define RANS_LOW (1u << 16)                /* lower end of the state range */
#define ESCAPE 255
#define ZERO_SYMBOL 127                    /* symbol of q = 0              */

/* ------------------------------------------------------------------------- */
/* IEEE binary16                                                             */
/* ------------------------------------------------------------------------- */

double plco_half_to_double(uint16_t h) {
  int sign = (h >> 15) & 1;
  int ex = (h >> 10) & 31;
  int man = h & 1023;
  double v;
  if (ex == 0) {
    v = ldexp((double)man, -24); /* zero and subnormals: man * 2^-24 */
  } else if (ex == 31) {
    v = man ? NAN : INFINITY;
  } else {
    v = ldexp((double)(1024 + man), ex - 25); /* (1 + man/1024) * 2^(ex-15) */
  }
  return sign ? -v : v;
}

uint16_t plco_double_to_half(double x) {
  uint16_t sign = signbit(x) ? 0x8000u : 0u;
  double a = fabs(x);
  if (isnan(x)) return (uint16_t)(sign | 0x7e00u);
  if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u); /* rounds past the largest finite value */
  if (a < ldexp(1.0, -14)) {
    /* subnormal range: multiples of 2^-24; nearbyint rounds half to even.
     * A result of 1024 is the smallest normal number, and its bit pattern
     * 0x0400 is what the plain integer gives. */
    double m = nearbyint(ldexp(a, 24));
    return (uint16_t)(sign | (uint16_t)m);
  }
  int e;
  (void)frexp(a, &e); /* a = f * 2^e, f in [0.5, 1) */
  int E = e - 1;      /* a = 1.xxx * 2^E            */
  double m = nearbyint(ldexp(a, 10 - E)); /* in [1024, 2048] */
  if (m >= 2048.0) {
    m = 1024.0;
    E += 1;
  }
  if (E + 15 >= 31) return (uint16_t)(sign | 0x7c00u);
  return (uint16_t)(sign | (uint16_t)((E + 15) << 10) | (uint16_t)((int)m - 1024));
}

/* ------------------------------------------------------------------------- */
/* Sec. 7.1: renormalised top-k weights                                      */
/* ------------------------------------------------------------------------- */

int plco_weights(const float *p, int k, int mode, double *w) {
  int j;
  if (k < 1) return PLCO_ERR_INVALID;
  for (j = 0; j < k; ++j) {
    if (isnan(p[j]) || p[j] < 0.0f) return PLCO_ERR_INVALID;
  }
  if (mode == PLCO_F32) {
    float Z = 0.0f;
    for (j = 0; j < k; ++j) Z = Z + p[j];
    if (!(Z > 0.0f) || !isfinite(Z)) return PLCO_ERR_INVALID;
    for (j = 0; j < k; ++j) {
      float wj = p[j] / Z;
      w[j] = (double)wj;
    }
  } else {
    double Z = 0.0;
    for (j = 0; j < k; ++j) Z = Z + (double)p[j];
    if (!(Z > 0.0) || !isfinite(Z)) return PLCO_ERR_INVALID;
    for (j = 0; j < k; ++j) w[j] = (double)p[j] / Z;
  }
  return PLCO_OK;
}

/* Weighted mean of the k candidates for one component (Sec. 7.1), j ascending. */
static double predict_one(const double *w, const uint16_t *cand, int64_t stride_j,
                          int k, int mode) {
  int j;
  if (mode == PLCO_F32) {
    float acc = 0.0f;
    for (j = 0; j < k; ++j) {
      float c = (float)plco_half_to_double(cand[(int64_t)j * stride_j]);
      acc = fmaf((float)w[j], c, acc);
    }
    return (double)acc;
  } else {
    double acc = 0.0;
    for (j = 0; j < k; ++j) {
      double c = plco_half_to_double(cand[(int64_t)j * stride_j]);
      acc = acc + w[j] * c;
    }
    return acc;
  }
}

static int check_dims(const plco_dims *dm) {
  if (!dm) return PLCO_ERR_INVALID;
  if (dm->S < 1 || dm->L < 1 || dm->H < 1 || dm->n < 1 || dm->d < 1) return PLCO_ERR_INVALID;
  if (dm->k < 1) return PLCO_ERR_INVALID;
  if (!(dm->delta > 0.0f) || !isfinite(dm->delta)) return PLCO_ERR_INVALID;
  if (dm->qmax < 1 || dm->qmax > 127) return PLCO_ERR_INVALID;
  return PLCO_OK;
}

/* ------------------------------------------------------------------------- */
/* Encode side: predict, subtract, quantise (Sec. 7.2, integration point 1)  */
/* ------------------------------------------------------------------------- */

/* Which prediction a position uses.  Without a `chosen` array every position
 * takes the weighted mean of Sec. 7.1.  With one, chosen[s*n+i] = j in [0,k)
 * says that the true token at the position is candidate j: by Lemma "KV
 * determinism" the KV vector is a function of the token prefix, so the
 * prediction is that candidate's vector itself; -1 says the token is not among
 * the candidates, and the weighted mean is used.  Returns -2 for any other value. */
static int position_choice(const int32_t *chosen, int64_t row, int k) {
  if (!chosen) return -1;
  int32_t j = chosen[row];
  if (j < -1 || j >= k) return -2;
  return (int)j;
}

/* Quantiser step of a position.  Without `bits` it is dm->delta everywhere.
 * With it (Def. "Surprisal-adaptive quantizer", Sec. 5.3: b_i bits per residual
 * component at position i; Cor. "Practical bit allocation", Sec. 9.4: b bits
 * mean a step of range / 2^b) the step is range * 2^-bits[s*n+i], an exact
 * scaling of the fp32 value `range` by a power of two.  Returns 0 for a bit
 * depth outside 1..PLCO_MAX_BITS. */
static float position_step(const plco_dims *dm, const uint8_t *bits, float range, int64_t row) {
  if (!bits) return dm->delta;
  int b = bits[row];
  if (b < 1 || b > PLCO_MAX_BITS) return 0.0f;
  return ldexpf(range, -b);
}

static int encode_positions(const plco_dims *dm, int mode,
                            const uint16_t *cand_k, const uint16_t *cand_v,
                            const float *probs, const int32_t *chosen,
                            const uint8_t *bits, float range,
                            const uint16_t *act_k, const uint16_t *act_v,
                            uint8_t *symbols, uint16_t *esc_vals, uint64_t esc_cap,
                            uint32_t *esc_cnt, uint64_t *esc_off,
                            double *pred_out, double *u_out) {
  int rc = check_dims(dm);
  if (rc) return rc;
  const int S = dm->S, L = dm->L, H = dm->H, n = dm->n, k = dm->k, d = dm->d;
  double w[64];
  if (k > 64) return PLCO_ERR_INVALID;
  uint64_t n_esc = 0; /* running length of the escape list over all streams */
  int64_t out = 0;    /* running index into symbols / pred_out / u_out      */

  for (int s = 0; s < S; ++s)
    for (int l = 0; l < L; ++l)
      for (int h = 0; h < H; ++h) {
        int64_t stream = ((int64_t)s * L + l) * H + h;
        esc_off[stream] = n_esc;
        uint32_t cnt = 0;
        for (int i = 0; i < n; ++i) {
          rc = plco_weights(probs + ((int64_t)s * n + i) * k, k, mode, w);
          if (rc) return rc;
          const int pick = position_choice(chosen, (int64_t)s * n + i, k);
          if (pick == -2) return PLCO_ERR_INVALID;
          const float step = position_step(dm, bits, range, (int64_t)s * n + i);
          if (!(step > 0.0f)) return PLCO_ERR_INVALID;
          for (int c = 0; c < 2; ++c) {
            const uint16_t *cand = c ? cand_v : cand_k;
            const uint16_t *act = c ? act_v : act_k;
            int64_t cbase = s * dm->cand_stride[0] + l * dm->cand_stride[1] +
                            h * dm->cand_stride[2] + i * dm->cand_stride[3];
            int64_t abase = s * dm->act_stride[0] + l * dm->act_stride[1] +
                            h * dm->act_stride[2] + i * dm->act_stride[3];
            for (int e = 0; e < d; ++e, ++out) {
              double pred = pick >= 0
                  ? plco_half_to_double(cand[cbase + (int64_t)pick * dm->cand_stride[4] + e])
                  : predict_one(w, cand + cbase + e, dm->cand_stride[4], k, mode);
              uint16_t raw = act[abase + e];
              double a = plco_half_to_double(raw);
              double u, q;
              if (mode == PLCO_F32) {
                float r = (float)a - (float)pred; /* Def. KV residual */
                float uf = r / step;
                u = (double)uf;
                q = (double)rintf(uf); /* round half to even */
              } else {
                double r = a - pred;
                u = r / (double)step;
                q = nearbyint(u);
              }
              if (pred_out) pred_out[out] = pred;
              if (u_out) u_out[out] = u;
              if (!isfinite(u) || fabs(q) > (double)dm->qmax) {
                symbols[out] = ESCAPE;
                if (n_esc >= esc_cap) return PLCO_ERR_CAPACITY;
                esc_vals[n_esc++] = raw;
                ++cnt;
              } else {
                symbols[out] = (uint8_t)((int)q + ZERO_SYMBOL);
              }
            }
          }
        }
        esc_cnt[stream] = cnt;
      }
  return PLCO_OK;
}

int plco_predict_residual(const plco_dims *dm, int mode,
                          const uint16_t *cand_k, const uint16_t *cand_v,
                          const float *probs,
                          const uint16_t *act_k, const uint16_t *act_v,
                          uint8_t *symbols, uint16_t *esc_vals, uint64_t esc_cap,
                          uint32_t *esc_cnt, uint64_t *esc_off,
                          double *pred_out, double *u_out) {
  return encode_positions(dm, mode, cand_k, cand_v, probs, NULL, NULL, 0.0f, act_k, act_v, symbols,
                          esc_vals, esc_cap, esc_cnt, esc_off, pred_out, u_out);
}

int plco_predict_residual_cond(const plco_dims *dm, int mode,
                               const uint16_t *cand_k, const uint16_t *cand_v,
                               const float *probs, const int32_t *chosen,
                               const uint16_t *act_k, const uint16_t *act_v,
                               uint8_t *symbols, uint16_t *esc_vals, uint64_t esc_cap,
                               uint32_t *esc_cnt, uint64_t *esc_off,
                               double *pred_out, double *u_out) {
  if (!chosen) return PLCO_ERR_INVALID;
  return encode_positions(dm, mode, cand_k, cand_v, probs, chosen, NULL, 0.0f, act_k, act_v, symbols,
                          esc_vals, esc_cap, esc_cnt, esc_off, pred_out, u_out);
}

int plco_predict_residual_adapt(const plco_dims *dm, int mode,
                                const uint16_t *cand_k, const uint16_t *cand_v,
                                const float *probs, const int32_t *chosen,
                                const uint8_t *bits, float range,
                                const uint16_t *act_k, const uint16_t *act_v,
                                uint8_t *symbols, uint16_t *esc_vals, uint64_t esc_cap,
                                uint32_t *esc_cnt, uint64_t *esc_off,
                                double *pred_out, double *u_out) {
  if (!chosen || !bits || !(range > 0.0f) || !isfinite(range)) return PLCO_ERR_INVALID;
  return encode_positions(dm, mode, cand_k, cand_v, probs, chosen, bits, range, act_k, act_v,
                          symbols, esc_vals, esc_cap, esc_cnt, esc_off, pred_out, u_out);
}

/* ------------------------------------------------------------------------- */
/* Symbol statistics                                                         */
/* ------------------------------------------------------------------------- */

int plco_histogram(const uint8_t *symbols, int64_t n_streams,
                   int64_t syms_per_stream, uint32_t *counts) {
  if (n_streams < 0 || syms_per_stream < 0) return PLCO_ERR_INVALID;
  for (int64_t st = 0; st < n_streams; ++st) {
    uint32_t *c = counts + st * 256;
    memset(c, 0, 256 * sizeof(uint32_t));
    for (int64_t t = 0; t < syms_per_stream; ++t) c[symbols[st * syms_per_stream + t]] += 1;
  }
  return PLCO_OK;
}

/* Frequencies on the 2^12 scale.  The cumulative counts are scaled and
 * floored, so differences sum to 4096 by construction; a symbol that occurs
 * but was scaled to zero then takes one unit from the currently largest
 * frequency (lowest symbol on ties), in ascending symbol order. */
int plco_build_freq(const uint32_t *counts, int64_t n_streams,
                    uint16_t *freq, uint16_t *cum) {
  for (int64_t st = 0; st < n_streams; ++st) {
    const uint32_t *cnt = counts + st * 256;
    uint32_t f[256];
    uint64_t T = 0, C = 0, prev = 0;
    int s;
    for (s = 0; s < 256; ++s) T += cnt[s];
    if (T == 0) return PLCO_ERR_INVALID;
    for (s = 0; s < 256; ++s) {
      C += cnt[s];
      uint64_t scaled = (C * RANS_SCALE) / T; /* floor(C[s+1] * 4096 / T) */
      f[s] = (uint32_t)(scaled - prev);
      prev = scaled;
    }
    for (s = 0; s < 256; ++s) {
      if (cnt[s] > 0 && f[s] == 0) {
        int donor = 0, m;
        for (m = 1; m < 256; ++m)
          if (f[m] > f[donor]) donor = m;
        f[donor] -= 1;
        f[s] = 1;
      }
    }
    uint32_t acc = 0;
    for (s = 0; s < 256; ++s) {
      freq[st * 256 + s] = (uint16_t)f[s];
      if (cum) cum[st * 257 + s] = (uint16_t)acc;
      acc += f[s];
    }
    if (cum) cum[st * 257 + 256] = (uint16_t)acc;
    if (acc != RANS_SCALE) return PLCO_ERR_INVALID;
  }
  return PLCO_OK;
}

/* ------------------------------------------------------------------------- */
/* 32-lane interleaved rANS                                                  */
/* ------------------------------------------------------------------------- */

int64_t plco_units_per_stream(int64_t syms_per_stream, int32_t chunk_syms) {
  if (chunk_syms <= 0) return 1;
  return (syms_per_stream + chunk_syms - 1) / chunk_syms;
}

/* Encode one unit.  Symbol t sits in lane t mod 32.  The encoder walks the
 * symbols from the last to the first so that the decoder meets them first to
 * last; words are appended in the order they are produced. */
static int rans_encode_unit(const uint8_t *sym, int64_t N, const uint16_t *f,
                            const uint32_t *cum, uint32_t *state_out,
                            uint16_t *words, uint64_t cap, uint32_t *n_words_out) {
  uint32_t x[RANS_LANES];
  uint64_t nw = 0;
  for (int lane = 0; lane < RANS_LANES; ++lane) x[lane] = RANS_LOW;
  for (int64_t t = N - 1; t >= 0; --t) { /* group descending, lane descending */
    int lane = (int)(t % RANS_LANES);
    uint32_t fs = f[sym[t]];
    uint32_t cs = cum[sym[t]];
    if (fs == 0) return PLCO_ERR_INVALID; /* symbol absent from the table */
    /* renormalise: keep the coding step's result below 2^32.  x >= fs * 2^20
     * is tested on the high bits because fs * 2^20 does not fit 32 bits for
     * fs = 4096.  One word always suffices. */
    if ((x[lane] >> 20) >= fs) {
      if (nw >= cap) return PLCO_ERR_CAPACITY;
      words[nw++] = (uint16_t)(x[lane] & 0xffffu);
      x[lane] >>= 16;
    }
    x[lane] = (x[lane] / fs) * RANS_SCALE + (x[lane] % fs) + cs;
  }
  for (int lane = 0; lane < RANS_LANES; ++lane) state_out[lane] = x[lane];
  if (nw > 0xffffffffull) return PLCO_ERR_CAPACITY;
  *n_words_out = (uint32_t)nw;
  return PLCO_OK;
}

/* Decode one unit: the exact inverse, symbols first to last, words consumed
 * from the end of the unit's word list backwards. */
static int rans_decode_unit(const uint16_t *f, const uint32_t *cum,
                            const uint8_t *slot_to_sym, const uint32_t *state_in,
                            const uint16_t *words, uint32_t n_words, int64_t N,
                            uint8_t *sym) {
  uint32_t x[RANS_LANES];
  uint64_t ptr = n_words;
  for (int lane = 0; lane < RANS_LANES; ++lane) x[lane] = state_in[lane];
  for (int64_t t = 0; t < N; ++t) { /* group ascending, lane ascending */
    int lane = (int)(t % RANS_LANES);
    uint32_t slot = x[lane] & (RANS_SCALE - 1);
    uint8_t s = slot_to_sym[slot];
    sym[t] = s;
    x[lane] = (uint32_t)f[s] * (x[lane] >> RANS_SCALE_BITS) + slot - cum[s];
    if (x[lane] < RANS_LOW) {
      if (ptr == 0) return PLCO_ERR_CORRUPT;
      x[lane] = (x[lane] << 16) | words[--ptr];
    }
  }
  /* integrity: every word used, every lane back at its initial state */
  if (ptr != 0) return PLCO_ERR_CORRUPT;
  for (int lane = 0; lane < RANS_LANES; ++lane)
    if (x[lane] != RANS_LOW) return PLCO_ERR_CORRUPT;
  return PLCO_OK;
}

static int check_rans_args(int64_t n_streams, int64_t N, int32_t chunk_syms) {
  if (n_streams < 0 || N < 1) return PLCO_ERR_INVALID;
  if (chunk_syms < 0 || (chunk_syms % RANS_LANES) != 0) return PLCO_ERR_INVALID;
  return PLCO_OK;
}

int plco_rans_encode(const uint8_t *symbols, int64_t n_streams,
                     int64_t syms_per_stream, int32_t chunk_syms,
                     const uint16_t *freq, uint32_t *states, uint16_t *words,
                     const uint64_t *word_off, uint64_t word_cap_per_unit,
                     uint32_t *n_words) {
  int rc = check_rans_args(n_streams, syms_per_stream, chunk_syms);
  if (rc) return rc;
  const int64_t N = syms_per_stream;
  const int64_t U = plco_units_per_stream(N, chunk_syms);
  const int64_t C = chunk_syms > 0 ? chunk_syms : N;
  for (int64_t st = 0; st < n_streams; ++st) {
    const uint16_t *f = freq + st * 256;
    uint32_t cum[257];
    cum[0] = 0;
    for (int s = 0; s < 256; ++s) cum[s + 1] = cum[s] + f[s];
    if (cum[256] != RANS_SCALE) return PLCO_ERR_INVALID;
    for (int64_t u = 0; u < U; ++u) {
      int64_t unit = st * U + u;
      int64_t begin = u * C;
      int64_t len = (begin + C <= N) ? C : (N - begin);
      rc = rans_encode_unit(symbols + st * N + begin, len, f, cum,
                            states + unit * RANS_LANES, words + word_off[unit],
                            word_cap_per_unit, n_words + unit);
      if (rc) return rc;
    }
  }
  return PLCO_OK;
}

int plco_rans_decode(const uint16_t *freq, const uint32_t *states,
                     const uint16_t *words, const uint64_t *word_off,
                     const uint32_t *n_words, int64_t n_streams,
                     int64_t syms_per_stream, int32_t chunk_syms,
                     uint8_t *symbols) {
  int rc = check_rans_args(n_streams, syms_per_stream, chunk_syms);
  if (rc) return rc;
  const int64_t N = syms_per_stream;
  const int64_t U = plco_units_per_stream(N, chunk_syms);
  const int64_t C = chunk_syms > 0 ? chunk_syms : N;
  for (int64_t st = 0; st < n_streams; ++st) {
    const uint16_t *f = freq + st * 256;
    uint32_t cum[257];
    uint8_t slot_to_sym[RANS_SCALE];
    cum[0] = 0;
    for (int s = 0; s < 256; ++s) cum[s + 1] = cum[s] + f[s];
    if (cum[256] != RANS_SCALE) return PLCO_ERR_CORRUPT;
    /* the symbol s with cum[s] <= slot < cum[s+1], tabulated for every slot */
    for (int s = 0; s < 256; ++s)
      for (uint32_t slot = cum[s]; slot < cum[s + 1]; ++slot) slot_to_sym[slot] = (uint8_t)s;
    for (int64_t u = 0; u < U; ++u) {
      int64_t unit = st * U + u;
      int64_t begin = u * C;
      int64_t len = (begin + C <= N) ? C : (N - begin);
      rc = rans_decode_unit(f, cum, slot_to_sym, states + unit * RANS_LANES,
                            words + word_off[unit], n_words[unit], len,
                            symbols + st * N + begin);
      if (rc) return rc;
    }
  }
  return PLCO_OK;
}

/* ------------------------------------------------------------------------- */
/* Decode side: dequantise, add the prediction back (Sec. 7.2, point 2)      */
/* ------------------------------------------------------------------------- */

static int decode_positions(const plco_dims *dm, int mode,
                            const uint16_t *cand_k, const uint16_t *cand_v,
                            const float *probs, const int32_t *chosen,
                            const uint8_t *bits, float range,
                            const uint8_t *symbols,
                            const uint16_t *esc_vals, const uint64_t *esc_off,
                            uint16_t *out_k, uint16_t *out_v, double *pre_round_out) {
  int rc = check_dims(dm);
  if (rc) return rc;
  const int S = dm->S, L = dm->L, H = dm->H, n = dm->n, k = dm->k, d = dm->d;
  double w[64];
  if (k > 64) return PLCO_ERR_INVALID;
  int64_t in = 0;

  for (int s = 0; s < S; ++s)
    for (int l = 0; l < L; ++l)
      for (int h = 0; h < H; ++h) {
        int64_t stream = ((int64_t)s * L + l) * H + h;
        uint64_t next_esc = esc_off[stream];
        for (int i = 0; i < n; ++i) {
          rc = plco_weights(probs + ((int64_t)s * n + i) * k, k, mode, w);
          if (rc) return rc;
          const int pick = position_choice(chosen, (int64_t)s * n + i, k);
          if (pick == -2) return PLCO_ERR_INVALID;
          const float step = position_step(dm, bits, range, (int64_t)s * n + i);
          if (!(step > 0.0f)) return PLCO_ERR_INVALID;
          for (int c = 0; c < 2; ++c) {
            const uint16_t *cand = c ? cand_v : cand_k;
            uint16_t *out = c ? out_v : out_k;
            int64_t cbase = s * dm->cand_stride[0] + l * dm->cand_stride[1] +
                            h * dm->cand_stride[2] + i * dm->cand_stride[3];
            int64_t abase = s * dm->act_stride[0] + l * dm->act_stride[1] +
                            h * dm->act_stride[2] + i * dm->act_stride[3];
            for (int e = 0; e < d; ++e, ++in) {
              uint8_t sym = symbols[in];
              if (sym == ESCAPE) {
                uint16_t raw = esc_vals[next_esc++];
                out[abase + e] = raw;
                if (pre_round_out) pre_round_out[in] = plco_half_to_double(raw);
                continue;
              }
              double pred = pick >= 0
                  ? plco_half_to_double(cand[cbase + (int64_t)pick * dm->cand_stride[4] + e])
                  : predict_one(w, cand + cbase + e, dm->cand_stride[4], k, mode);
              int q = (int)sym - ZERO_SYMBOL;
              double xhat;
              if (mode == PLCO_F32) {
                xhat = (double)fmaf((float)q, step, (float)pred);
              } else {
                xhat = pred + (double)q * (double)step;
              }
              if (pre_round_out) pre_round_out[in] = xhat;
              out[abase + e] = plco_double_to_half(xhat);
            }
          }
        }
      }
  return PLCO_OK;
}

int plco_reconstruct(const plco_dims *dm, int mode,
                     const uint16_t *cand_k, const uint16_t *cand_v,
                     const float *probs, const uint8_t *symbols,
                     const uint16_t *esc_vals, const uint64_t *esc_off,
                     uint16_t *out_k, uint16_t *out_v, double *pre_round_out) {
  return decode_positions(dm, mode, cand_k, cand_v, probs, NULL, NULL, 0.0f, symbols, esc_vals,
                          esc_off, out_k, out_v, pre_round_out);
}

int plco_reconstruct_cond(const plco_dims *dm, int mode,
                          const uint16_t *cand_k, const uint16_t *cand_v,
                          const float *probs, const int32_t *chosen,
                          const uint8_t *symbols,
                          const uint16_t *esc_vals, const uint64_t *esc_off,
                          uint16_t *out_k, uint16_t *out_v, double *pre_round_out) {
  if (!chosen) return PLCO_ERR_INVALID;
  return decode_positions(dm, mode, cand_k, cand_v, probs, chosen, NULL, 0.0f, symbols, esc_vals,
                          esc_off, out_k, out_v, pre_round_out);
}

int plco_reconstruct_adapt(const plco_dims *dm, int mode,
                           const uint16_t *cand_k, const uint16_t *cand_v,
                           const float *probs, const int32_t *chosen,
                           const uint8_t *bits, float range, const uint8_t *symbols,
                           const uint16_t *esc_vals, const uint64_t *esc_off,
                           uint16_t *out_k, uint16_t *out_v, double *pre_round_out) {
  if (!chosen || !bits || !(range > 0.0f) || !isfinite(range)) return PLCO_ERR_INVALID;
  return decode_positions(dm, mode, cand_k, cand_v, probs, chosen, bits, range, symbols, esc_vals,
                          esc_off, out_k, out_v, pre_round_out);
}

/* ------------------------------------------------------------------------- */
/* Token-conditional coding: which candidate is the true token, and the code  */
/* of that index under the model's own probabilities (Thm. "Sequential       */
/* entropy bound": the cost of a position is at most the token's surprisal)  */
/* ------------------------------------------------------------------------- */

/* The candidate whose layer-0, head-0 key row is nearest (squared distance,
 * components ascending) to the actual one; lowest index on ties; a distance
 * that is NaN never wins.  If the nearest is farther than max_mean_sq per
 * component, or none compares, the position is a miss (-1). */
int plco_select_candidate(const plco_dims *dm, int mode, const uint16_t *cand_k,
                          const uint16_t *act_k, float max_mean_sq, int32_t *chosen) {
  int rc = check_dims(dm);
  if (rc) return rc;
  const int S = dm->S, n = dm->n, k = dm->k, d = dm->d;
  for (int s = 0; s < S; ++s)
    for (int i = 0; i < n; ++i) {
      int64_t cbase = s * dm->cand_stride[0] + i * dm->cand_stride[3]; /* l = 0, h = 0 */
      int64_t abase = s * dm->act_stride[0] + i * dm->act_stride[3];
      int best_j = -1;
      double best = 0.0;
      for (int j = 0; j < k; ++j) {
        double D;
        if (mode == PLCO_F32) {
          float acc = 0.0f;
          for (int e = 0; e < d; ++e) {
            float a = (float)plco_half_to_double(act_k[abase + e]);
            float c = (float)plco_half_to_double(cand_k[cbase + (int64_t)j * dm->cand_stride[4] + e]);
            float diff = a - c;
            acc = fmaf(diff, diff, acc);
          }
          D = (double)acc;
        } else {
          double acc = 0.0;
          for (int e = 0; e < d; ++e) {
            double a = plco_half_to_double(act_k[abase + e]);
            double c = plco_half_to_double(cand_k[cbase + (int64_t)j * dm->cand_stride[4] + e]);
            acc = acc + (a - c) * (a - c);
          }
          D = acc;
        }
        if (best_j < 0 ? (D == D) : (D < best)) {
          best_j = j;
          best = D;
        }
      }
      double limit = (mode == PLCO_F32) ? (double)(max_mean_sq * (float)d)
                                        : (double)max_mean_sq * (double)d;
      if (best_j >= 0 && !(best <= limit)) best_j = -1;
      chosen[(int64_t)s * n + i] = best_j;
    }
  return PLCO_OK;
}

/* Frequencies of the k + 1 index symbols of one position on the 2^12 scale:
 * symbol j < k is "the token is candidate j", symbol k is "none of them" and
 * owns the mass the k probabilities leave.  Boundaries are the floored, scaled
 * running sums of the raw probabilities in single precision (c = c + p_j, j
 * ascending), clipped at 4096; then every symbol that got nothing takes one
 * unit from the currently largest (lowest index on ties), j ascending, so that
 * each of the k + 1 symbols can be coded. */
int plco_index_table(const float *p, int k, uint16_t *f) {
  uint32_t fr[PLCO_MAX_K + 1];
  uint32_t prev = 0;
  float c = 0.0f;
  int j;
  if (k < 1 || k > PLCO_MAX_K) return PLCO_ERR_INVALID;
  for (j = 0; j < k; ++j)
    if (isnan(p[j]) || p[j] < 0.0f) return PLCO_ERR_INVALID;
  for (j = 0; j < k; ++j) {
    c = c + p[j];
    float scaled = floorf(c * 4096.0f);
    if (!(scaled < 4096.0f)) scaled = 4096.0f;
    uint32_t b = (uint32_t)scaled;
    fr[j] = b - prev;
    prev = b;
  }
  fr[k] = RANS_SCALE - prev;
  for (j = 0; j <= k; ++j) {
    if (fr[j] == 0) {
      int donor = 0, m;
      for (m = 1; m <= k; ++m)
        if (fr[m] > fr[donor]) donor = m;
      fr[donor] -= 1;
      fr[j] = 1;
    }
  }
  for (j = 0; j <= k; ++j) f[j] = (uint16_t)fr[j];
  return PLCO_OK;
}

/* The index stream of a session: one symbol per position (chosen, or k for
 * -1), coded with the same 32-lane rANS as the residuals (position i in lane
 * i mod 32, last position first, words in emission order), except that every
 * position has its own table. */
int plco_index_encode(const float *probs, const int32_t *chosen, int32_t S, int32_t n,
                      int32_t k, uint32_t *states, uint16_t *words,
                      const uint64_t *word_off, uint64_t word_cap, uint32_t *n_words) {
  if (S < 0 || n < 1 || k < 1 || k > PLCO_MAX_K) return PLCO_ERR_INVALID;
  for (int s = 0; s < S; ++s) {
    uint32_t x[RANS_LANES];
    uint16_t *out = words + word_off[s];
    uint64_t nw = 0;
    for (int lane = 0; lane < RANS_LANES; ++lane) x[lane] = RANS_LOW;
    for (int i = n - 1; i >= 0; --i) {
      int64_t row = (int64_t)s * n + i;
      uint16_t f[PLCO_MAX_K + 1];
      int rc = plco_index_table(probs + row * k, k, f);
      if (rc) return rc;
      int32_t j = chosen[row];
      if (j < -1 || j >= k) return PLCO_ERR_INVALID;
      int sym = j < 0 ? k : j;
      uint32_t fs = f[sym], cs = 0;
      for (int m = 0; m < sym; ++m) cs += f[m];
      int lane = i % RANS_LANES;
      if ((x[lane] >> 20) >= fs) {
        if (nw >= word_cap) return PLCO_ERR_CAPACITY;
        out[nw++] = (uint16_t)(x[lane] & 0xffffu);
        x[lane] >>= 16;
      }
      x[lane] = (x[lane] / fs) * RANS_SCALE + (x[lane] % fs) + cs;
    }
    for (int lane = 0; lane < RANS_LANES; ++lane) states[(int64_t)s * RANS_LANES + lane] = x[lane];
    n_words[s] = (uint32_t)nw;
  }
  return PLCO_OK;
}

int plco_index_decode(const float *probs, const uint32_t *states, const uint16_t *words,
                      const uint64_t *word_off, const uint32_t *n_words, int32_t S,
                      int32_t n, int32_t k, int32_t *chosen) {
  if (S < 0 || n < 1 || k < 1 || k > PLCO_MAX_K) return PLCO_ERR_INVALID;
  for (int s = 0; s < S; ++s) {
    uint32_t x[RANS_LANES];
    const uint16_t *in = words + word_off[s];
    uint64_t ptr = n_words[s];
    for (int lane = 0; lane < RANS_LANES; ++lane) x[lane] = states[(int64_t)s * RANS_LANES + lane];
    for (int i = 0; i < n; ++i) {
      int64_t row = (int64_t)s * n + i;
      uint16_t f[PLCO_MAX_K + 1];
      int rc = plco_index_table(probs + row * k, k, f);
      if (rc) return rc;
      int lane = i % RANS_LANES;
      uint32_t slot = x[lane] & (RANS_SCALE - 1);
      uint32_t cs = 0;
      int sym = 0;
      while (cs + f[sym] <= slot) { /* the symbol whose interval holds the slot */
        cs += f[sym];
        ++sym;
      }
      chosen[row] = sym == k ? -1 : sym;
      x[lane] = (uint32_t)f[sym] * (x[lane] >> RANS_SCALE_BITS) + slot - cs;
      if (x[lane] < RANS_LOW) {
        if (ptr == 0) return PLCO_ERR_CORRUPT;
        x[lane] = (x[lane] << 16) | in[--ptr];
      }
    }
    if (ptr != 0) return PLCO_ERR_CORRUPT;
    for (int lane = 0; lane < RANS_LANES; ++lane)
      if (x[lane] != RANS_LOW) return PLCO_ERR_CORRUPT;
  }
  return PLCO_OK;
}

/* ------------------------------------------------------------------------- */
/* Surprisal-adaptive quantiser (Sec. 5.3) with one table per bit depth       */
/* ------------------------------------------------------------------------- */

/* b_i = min(bmax, max(1, floor(b0 * h_i / hbar))) with h_i the position's coded
 * surprisal log2(4096 / f), f the index-table frequency of its token (symbol k
 * for a miss).  floor(b0 * h / hbar) >= m  <=>  f <= 4096 * 2^(-m * hbar / b0),
 * so the depth is a count of integer comparisons against the thresholds
 * thr[m] = floor(4096 * 2^(-m * hbar / b0)), m = 2..bmax (thr[0], thr[1] unused),
 * which plco_surprisal_thresholds derives from b0 and hbar.  The definition has no
 * upper limit on b_i; bmax is the caller's, up to what this file's arrays hold
 * (PLCO_MAX_BITS). */
int plco_surprisal_thresholds(double b0, double hbar, int32_t bmax, uint16_t *thr) {
  if (!(b0 > 0.0) || !(hbar > 0.0) || bmax < 1 || bmax > PLCO_MAX_BITS || !thr) return PLCO_ERR_INVALID;
  thr[0] = thr[1] = 0;
  for (int m = 2; m <= bmax; ++m) {
    double t = floor(4096.0 * pow(2.0, -(double)m * hbar / b0));
    if (t < 0.0) t = 0.0;
    if (t > 4096.0) t = 4096.0;
    thr[m] = (uint16_t)t;
  }
  return PLCO_OK;
}

int plco_surprisal_bits(const float *probs, const int32_t *chosen, int32_t S, int32_t n,
                        int32_t k, const uint16_t *thr, int32_t bmax, uint8_t *bits) {
  if (S < 0 || n < 1 || k < 1 || k > PLCO_MAX_K || bmax < 1 || bmax > PLCO_MAX_BITS)
    return PLCO_ERR_INVALID;
  for (int64_t row = 0; row < (int64_t)S * n; ++row) {
    uint16_t f[PLCO_MAX_K + 1];
    int rc = plco_index_table(probs + row * k, k, f);
    if (rc) return rc;
    int32_t j = chosen[row];
    if (j < -1 || j >= k) return PLCO_ERR_INVALID;
    uint32_t fs = f[j < 0 ? k : j];
    int b = 1;
    for (int m = 2; m <= bmax; ++m)
      if (fs <= thr[m]) b = m;
    bits[row] = (uint8_t)b;
  }
  return PLCO_OK;
}

/* Counts per (stream, bit depth): counts[(stream * n_tables + b - 1) * 256 + sym].
 * Stream st belongs to session st / streams_per_session; symbol t of a stream
 * belongs to position t / syms_per_pos. */
int plco_histogram_bucketed(const uint8_t *symbols, int64_t n_streams, int64_t syms_per_stream,
                            int32_t syms_per_pos, int32_t streams_per_session,
                            const uint8_t *bits, int32_t n_tables, uint32_t *counts) {
  if (n_streams < 0 || syms_per_stream < 1 || syms_per_pos < 1 || streams_per_session < 1 ||
      n_tables < 1 || n_tables > PLCO_MAX_BITS || syms_per_stream % syms_per_pos)
    return PLCO_ERR_INVALID;
  const int64_t n = syms_per_stream / syms_per_pos;
  memset(counts, 0, (size_t)n_streams * n_tables * 256 * sizeof(uint32_t));
  for (int64_t st = 0; st < n_streams; ++st)
    for (int64_t t = 0; t < syms_per_stream; ++t) {
      int b = bits[(st / streams_per_session) * n + t / syms_per_pos];
      if (b < 1 || b > n_tables) return PLCO_ERR_INVALID;
      counts[(st * n_tables + (b - 1)) * 256 + symbols[st * syms_per_stream + t]] += 1;
    }
  return PLCO_OK;
}

/* Frequency tables for rows of counts where a row may be empty (a bit depth
 * that does not occur in a stream): such a row gets all-zero frequencies. */
int plco_build_freq_sparse(const uint32_t *counts, int64_t n_rows, uint16_t *freq) {
  for (int64_t r = 0; r < n_rows; ++r) {
    uint64_t T = 0;
    for (int s = 0; s < 256; ++s) T += counts[r * 256 + s];
    if (T == 0) {
      memset(freq + r * 256, 0, 256 * sizeof(uint16_t));
    } else {
      int rc = plco_build_freq(counts + r * 256, 1, freq + r * 256, NULL);
      if (rc) return rc;
    }
  }
  return PLCO_OK;
}

/* rANS as above, except that symbol t of a stream is coded with the table of
 * its position's bit depth: freq[(stream * n_tables + b - 1) * 256 + sym]. */
static int bucket_of(const uint8_t *bits, int64_t st, int64_t t, int64_t n, int32_t syms_per_pos,
                     int32_t streams_per_session, int32_t n_tables) {
  int b = bits[(st / streams_per_session) * n + t / syms_per_pos];
  return (b < 1 || b > n_tables) ? -1 : b - 1;
}

int plco_rans_encode_bucketed(const uint8_t *symbols, int64_t n_streams, int64_t syms_per_stream,
                              int32_t chunk_syms, int32_t syms_per_pos,
                              int32_t streams_per_session, const uint8_t *bits, int32_t n_tables,
                              const uint16_t *freq, uint32_t *states, uint16_t *words,
                              const uint64_t *word_off, uint64_t word_cap_per_unit,
                              uint32_t *n_words) {
  int rc = check_rans_args(n_streams, syms_per_stream, chunk_syms);
  if (rc) return rc;
  if (syms_per_pos < 1 || syms_per_stream % syms_per_pos || n_tables < 1 || n_tables > PLCO_MAX_BITS)
    return PLCO_ERR_INVALID;
  const int64_t N = syms_per_stream, n = N / syms_per_pos;
  const int64_t U = plco_units_per_stream(N, chunk_syms);
  const int64_t C = chunk_syms > 0 ? chunk_syms : N;
  for (int64_t st = 0; st < n_streams; ++st) {
    uint32_t cum[PLCO_MAX_BITS][257];
    for (int b = 0; b < n_tables; ++b) {
      const uint16_t *f = freq + (st * n_tables + b) * 256;
      cum[b][0] = 0;
      for (int s = 0; s < 256; ++s) cum[b][s + 1] = cum[b][s] + f[s];
      if (cum[b][256] != RANS_SCALE && cum[b][256] != 0) return PLCO_ERR_INVALID;
    }
    for (int64_t u = 0; u < U; ++u) {
      int64_t unit = st * U + u, begin = u * C;
      int64_t len = (begin + C <= N) ? C : (N - begin);
      uint32_t x[RANS_LANES];
      uint16_t *out = words + word_off[unit];
      uint64_t nw = 0;
      for (int lane = 0; lane < RANS_LANES; ++lane) x[lane] = RANS_LOW;
      for (int64_t t = len - 1; t >= 0; --t) {
        int lane = (int)(t % RANS_LANES);
        int b = bucket_of(bits, st, begin + t, n, syms_per_pos, streams_per_session, n_tables);
        if (b < 0) return PLCO_ERR_INVALID;
        uint8_t sym = symbols[st * N + begin + t];
        uint32_t fs = freq[(st * n_tables + b) * 256 + sym], cs = cum[b][sym];
        if (fs == 0) return PLCO_ERR_INVALID;
        if ((x[lane] >> 20) >= fs) {
          if (nw >= word_cap_per_unit) return PLCO_ERR_CAPACITY;
          out[nw++] = (uint16_t)(x[lane] & 0xffffu);
          x[lane] >>= 16;
        }
        x[lane] = (x[lane] / fs) * RANS_SCALE + (x[lane] % fs) + cs;
      }
      for (int lane = 0; lane < RANS_LANES; ++lane) states[unit * RANS_LANES + lane] = x[lane];
      n_words[unit] = (uint32_t)nw;
    }
  }
  return PLCO_OK;
}

int plco_rans_decode_bucketed(const uint16_t *freq, const uint32_t *states, const uint16_t *words,
                              const uint64_t *word_off, const uint32_t *n_words,
                              int64_t n_streams, int64_t syms_per_stream, int32_t chunk_syms,
                              int32_t syms_per_pos, int32_t streams_per_session,
                              const uint8_t *bits, int32_t n_tables, uint8_t *symbols) {
  int rc = check_rans_args(n_streams, syms_per_stream, chunk_syms);
  if (rc) return rc;
  if (syms_per_pos < 1 || syms_per_stream % syms_per_pos || n_tables < 1 || n_tables > PLCO_MAX_BITS)
    return PLCO_ERR_INVALID;
  const int64_t N = syms_per_stream, n = N / syms_per_pos;
  const int64_t U = plco_units_per_stream(N, chunk_syms);
  const int64_t C = chunk_syms > 0 ? chunk_syms : N;
  for (int64_t st = 0; st < n_streams; ++st) {
    for (int64_t u = 0; u < U; ++u) {
      int64_t unit = st * U + u, begin = u * C;
      int64_t len = (begin + C <= N) ? C : (N - begin);
      uint32_t x[RANS_LANES];
      const uint16_t *in = words + word_off[unit];
      uint64_t ptr = n_words[unit];
      for (int lane = 0; lane < RANS_LANES; ++lane) x[lane] = states[unit * RANS_LANES + lane];
      for (int64_t t = 0; t < len; ++t) {
        int lane = (int)(t % RANS_LANES);
        int b = bucket_of(bits, st, begin + t, n, syms_per_pos, streams_per_session, n_tables);
        if (b < 0) return PLCO_ERR_INVALID;
        const uint16_t *f = freq + (st * n_tables + b) * 256;
        uint32_t slot = x[lane] & (RANS_SCALE - 1), cs = 0;
        int sym = 0;
        while (sym < 256 && cs + f[sym] <= slot) { /* the symbol whose interval holds the slot */
          cs += f[sym];
          ++sym;
        }
        if (sym == 256) return PLCO_ERR_CORRUPT; /* empty table */
        symbols[st * N + begin + t] = (uint8_t)sym;
        x[lane] = (uint32_t)f[sym] * (x[lane] >> RANS_SCALE_BITS) + slot - cs;
        if (x[lane] < RANS_LOW) {
          if (ptr == 0) return PLCO_ERR_CORRUPT;
          x[lane] = (x[lane] << 16) | in[--ptr];
        }
      }
      if (ptr != 0) return PLCO_ERR_CORRUPT;
      for (int lane = 0; lane < RANS_LANES; ++lane)
        if (x[lane] != RANS_LOW) return PLCO_ERR_CORRUPT;
    }
  }
  return PLCO_OK;
}
