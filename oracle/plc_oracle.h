/*
 * plc_oracle.h -- CPU oracle for predictive delta coding of a KV cache.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, single-threaded C
 * implementation of what the coding path computes.  It exists so that tests
 * and the benchmark's CPU-baseline leg have something obviously correct to
 * compare against.  It shares no code, header, table or helper with the GPU
 * library and must never be called from a product path.
 *
 * What it follows (section / definition names are the paper's):
 *   - Sec. 7.1 "Top-k approximation": the predicted KV vector is the
 *     probability-weighted mean of k candidate KV vectors, with the k
 *     probabilities renormalised to sum to one.
 *   - Def. "KV residual" (Sec. 5.2): R_i = KV_i - predicted KV_i.
 *   - Sec. 7.2 "Integration with the inference loop": before a write, predict,
 *     subtract, quantise, store; before a read, dequantise and add the
 *     identically recomputed prediction back.
 *   - Prop. "Three-layer composition" (Sec. 6.2), correctness paragraph: the
 *     error of the recovered KV equals the quantiser's error on the residual.
 *   - Cor. "Practical bit allocation" (Sec. 9.4): a uniform quantiser of step
 *     Delta has distortion about Delta^2 / 12.
 *   - Prop. "Layer orthogonality", proof (Sec. 6.1): the residual is stored with a
 *     code of length about its entropy "by standard source coding".
 *
 * The paper fixes neither an alphabet nor an entropy coder.  The concrete
 * format implemented here (and documented at each function) is:
 *   symbols   one byte per KV component: q + 127 for q = round(R / Delta) in
 *             [-qmax, qmax]; 255 = escape, whose raw fp16 bit pattern goes to
 *             a per-stream side list in symbol order;
 *   streams   one per (session, layer, KV head); symbol index inside a stream
 *             t = (i * 2 + c) * d + e  (position i, c = 0 for K / 1 for V,
 *             component e), so a stream has N = 2 n d symbols;
 *   tables    integer frequencies summing to 2^12 per stream;
 *   coder     32 interleaved rANS lanes per stream, 32-bit states kept in
 *             [2^16, 2^32), 16-bit renormalisation words.
 *
 * Arithmetic: PLCO_F64 evaluates the floating-point steps in double
 * precision.  PLCO_F32 evaluates them in strict single precision in a fixed
 * operation order (no reassociation, fused multiply-add where stated), which
 * is the precision a single-precision device kernel takes its rounding
 * decisions in.
 *
 * Pins (tests/ -m "not gpu"): one-hot / k = 1 gives all-zero residuals; the
 * reconstruction error is at most Delta/2 and its mean square is Delta^2/12;
 * E|R|^2 equals the candidate variance under the predictive distribution plus
 * the noise; symbol entropy matches the closed-form Gaussian-mixture pmf of
 * the synthetic workload; frequency tables match closed forms; rANS
 * round-trips on brute-force edge cases, matches a hand-worked example and
 * obeys the size law against the table's cross entropy.
 * Token-conditional functions: all positions marked "not a candidate" reduce
 * to the functions above bit for bit; a chosen candidate equals the weighted
 * mean under a one-hot row; noise-free actual vectors give all-zero residuals;
 * symbol entropy matches the closed-form pmf of a quantised Gaussian; index
 * tables match closed forms for dyadic rows; the index stream's length obeys
 * the size law against the tokens' surprisal and a hand-worked example.
 * Adaptive quantiser functions: one bit depth everywhere reduces to the fixed
 * step functions bit for bit (and one table to the plain histogram, table and
 * rANS functions); bit depths match the floating formula of the definition on
 * every frequency; error at most half the position's step; per-depth symbol
 * statistics match the closed-form pmf.
 * Parity unpinned: the exact bit layout of the rANS streams is this format's
 * own definition, so agreement with any external coder is not sought.
 */
#ifndef PLC_ORACLE_H
#define PLC_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  PLCO_OK = 0,
  PLCO_ERR_INVALID = 1,   /* bad argument or invalid probability row        */
  PLCO_ERR_CAPACITY = 2,  /* an output list is too small                    */
  PLCO_ERR_CORRUPT = 3    /* decoder integrity check failed                 */
};

enum { PLCO_F64 = 0, PLCO_F32 = 1 };

typedef struct plco_dims {
  int32_t S, L, H, n, k, d;
  int64_t cand_stride[5]; /* element strides for (s, l, h, i, j); e is contiguous */
  int64_t act_stride[4];  /* element strides for (s, l, h, i);    e is contiguous */
  float delta;            /* quantiser step; THE step is this fp32 value    */
  int32_t qmax;           /* largest |q| that has its own symbol, <= 127    */
} plco_dims;

/* IEEE binary16 <-> double, round to nearest even, subnormals kept. */
double plco_half_to_double(uint16_t h);
uint16_t plco_double_to_half(double x);

/* Renormalised top-k weights of one probability row (Sec. 7.1).
 * w[j] = p[j] / sum_m p[m].  Rows with a negative or NaN entry, or a sum that
 * is not a positive finite number, are invalid.  mode selects double or
 * strict-float arithmetic; the result is returned in double either way. */
int plco_weights(const float *p, int k, int mode, double *w);

/* Encode side, floating-point part (Sec. 7.1, Def. KV residual, Sec. 7.2 (1)).
 * cand_k / cand_v: fp16 bit patterns, logical [S,L,H,n,k,d] with the given strides.
 * probs: fp32 [S,n,k] raw top-k probabilities (one row per session and position,
 *        shared by every layer, head, K and V).
 * act_k / act_v: fp16 bit patterns, logical [S,L,H,n,d].
 * symbols: u8 [S,L,H,n,2,d].  esc_vals: u16 list, stream after stream, each
 * stream's escapes in symbol order; esc_off[stream] is where a stream's list
 * starts and esc_cnt[stream] its length.  pred_out (nullable): the prediction,
 * double [S,L,H,n,2,d].  u_out (nullable): R / Delta before rounding, same shape. */
int plco_predict_residual(const plco_dims *dm, int mode,
                          const uint16_t *cand_k, const uint16_t *cand_v,
                          const float *probs,
                          const uint16_t *act_k, const uint16_t *act_v,
                          uint8_t *symbols, uint16_t *esc_vals, uint64_t esc_cap,
                          uint32_t *esc_cnt, uint64_t *esc_off,
                          double *pred_out, double *u_out);

/* Per-stream 256-bin symbol counts. counts: u32 [n_streams, 256]. */
int plco_histogram(const uint8_t *symbols, int64_t n_streams,
                   int64_t syms_per_stream, uint32_t *counts);

/* Counts -> integer frequencies summing to 4096 with f > 0 iff count > 0.
 * freq: u16 [n_streams,256]; cum (nullable): u16 [n_streams,257]. */
int plco_build_freq(const uint32_t *counts, int64_t n_streams,
                    uint16_t *freq, uint16_t *cum);

/* Number of independently coded units per stream for a chunk length. */
int64_t plco_units_per_stream(int64_t syms_per_stream, int32_t chunk_syms);

/* 32-lane interleaved rANS.  chunk_syms = 0 codes each stream as one unit;
 * otherwise (a multiple of 32) each run of chunk_syms symbols is its own unit
 * with the stream's table.  Unit index = stream * units_per_stream + chunk.
 * states: u32 [n_units,32]; unit u writes words[word_off[u] .. +n_words[u]). */
int plco_rans_encode(const uint8_t *symbols, int64_t n_streams,
                     int64_t syms_per_stream, int32_t chunk_syms,
                     const uint16_t *freq, uint32_t *states, uint16_t *words,
                     const uint64_t *word_off, uint64_t word_cap_per_unit,
                     uint32_t *n_words);

int plco_rans_decode(const uint16_t *freq, const uint32_t *states,
                     const uint16_t *words, const uint64_t *word_off,
                     const uint32_t *n_words, int64_t n_streams,
                     int64_t syms_per_stream, int32_t chunk_syms,
                     uint8_t *symbols);

/* Decode side, floating-point part (Sec. 7.2 (2)): prediction recomputed from
 * the same candidates and probabilities, plus the dequantised residual,
 * rounded to fp16; escapes restored bit for bit from the side list. */
int plco_reconstruct(const plco_dims *dm, int mode,
                     const uint16_t *cand_k, const uint16_t *cand_v,
                     const float *probs, const uint8_t *symbols,
                     const uint16_t *esc_vals, const uint64_t *esc_off,
                     uint16_t *out_k, uint16_t *out_v, double *pre_round_out);

/* ---- Token-conditional coding (Lemma "KV determinism", Thm. "Sequential entropy bound") ----
 * Given the token, the KV vector is determined; so when the true token is one
 * of the k candidates the prediction is that candidate's vector and only the
 * index has to be paid for, at about the token's surprisal.
 *
 * chosen: i32 [S,n]; j in [0,k) = the true token is candidate j (prediction =
 * candidate j, exactly); -1 = not among the candidates (prediction = the
 * weighted mean, as in plco_predict_residual).  Everything else as in the
 * functions without the suffix. */
#define PLCO_MAX_K 32

int plco_predict_residual_cond(const plco_dims *dm, int mode,
                               const uint16_t *cand_k, const uint16_t *cand_v,
                               const float *probs, const int32_t *chosen,
                               const uint16_t *act_k, const uint16_t *act_v,
                               uint8_t *symbols, uint16_t *esc_vals, uint64_t esc_cap,
                               uint32_t *esc_cnt, uint64_t *esc_off,
                               double *pred_out, double *u_out);

int plco_reconstruct_cond(const plco_dims *dm, int mode,
                          const uint16_t *cand_k, const uint16_t *cand_v,
                          const float *probs, const int32_t *chosen,
                          const uint8_t *symbols,
                          const uint16_t *esc_vals, const uint64_t *esc_off,
                          uint16_t *out_k, uint16_t *out_v, double *pre_round_out);

/* Encoder-side recovery of `chosen` from the vectors alone: per (s, i), the
 * candidate whose key row in layer 0, head 0 is nearest to the actual one in
 * squared distance (components ascending; F32: diff in fp32, fused
 * multiply-add accumulate); -1 if that distance exceeds max_mean_sq * d. */
int plco_select_candidate(const plco_dims *dm, int mode, const uint16_t *cand_k,
                          const uint16_t *act_k, float max_mean_sq, int32_t *chosen);

/* Frequencies (sum 4096, all >= 1) of the k+1 index symbols of one position
 * from its raw top-k probabilities; symbol k = "not among the candidates". */
int plco_index_table(const float *p, int k, uint16_t *f);

/* One 32-lane rANS unit per session over the n index symbols, each coded with
 * its own position's table.  states: u32 [S,32]; session s writes
 * words[word_off[s] .. +n_words[s]). */
int plco_index_encode(const float *probs, const int32_t *chosen, int32_t S, int32_t n,
                      int32_t k, uint32_t *states, uint16_t *words,
                      const uint64_t *word_off, uint64_t word_cap, uint32_t *n_words);

int plco_index_decode(const float *probs, const uint32_t *states, const uint16_t *words,
                      const uint64_t *word_off, const uint32_t *n_words, int32_t S,
                      int32_t n, int32_t k, int32_t *chosen);

/* ---- Surprisal-adaptive quantiser (Def. in Sec. 5.3; Cor. "Practical bit allocation") ----
 * bits: u8 [S,n], b_i in 1..PLCO_MAX_BITS; the quantiser step of position i is
 * range * 2^-b_i (range: fp32 > 0, scaled exactly).  chosen as above (all -1
 * = weighted mean everywhere).  Symbols of positions with depth b are counted
 * and coded with the stream's table number b - 1. */
#define PLCO_MAX_BITS 16 /* bound of this file's per-depth arrays; the definition itself has none */

int plco_predict_residual_adapt(const plco_dims *dm, int mode,
                                const uint16_t *cand_k, const uint16_t *cand_v,
                                const float *probs, const int32_t *chosen,
                                const uint8_t *bits, float range,
                                const uint16_t *act_k, const uint16_t *act_v,
                                uint8_t *symbols, uint16_t *esc_vals, uint64_t esc_cap,
                                uint32_t *esc_cnt, uint64_t *esc_off,
                                double *pred_out, double *u_out);

int plco_reconstruct_adapt(const plco_dims *dm, int mode,
                           const uint16_t *cand_k, const uint16_t *cand_v,
                           const float *probs, const int32_t *chosen,
                           const uint8_t *bits, float range, const uint8_t *symbols,
                           const uint16_t *esc_vals, const uint64_t *esc_off,
                           uint16_t *out_k, uint16_t *out_v, double *pre_round_out);

/* Bit depth per position from the token's coded surprisal and integer
 * thresholds thr[2..bmax] (non-increasing): b = the largest m with f <= thr[m], else 1. */
/* thr[m] = floor(4096 * 2^(-m * hbar / b0)) for m = 2..bmax; thr[0] = thr[1] = 0 (host array of
 * bmax + 1 entries).  b0, hbar > 0. */
int plco_surprisal_thresholds(double b0, double hbar, int32_t bmax, uint16_t *thr);

int plco_surprisal_bits(const float *probs, const int32_t *chosen, int32_t S, int32_t n,
                        int32_t k, const uint16_t *thr, int32_t bmax, uint8_t *bits);

int plco_histogram_bucketed(const uint8_t *symbols, int64_t n_streams, int64_t syms_per_stream,
                            int32_t syms_per_pos, int32_t streams_per_session,
                            const uint8_t *bits, int32_t n_tables, uint32_t *counts);

int plco_build_freq_sparse(const uint32_t *counts, int64_t n_rows, uint16_t *freq);

int plco_rans_encode_bucketed(const uint8_t *symbols, int64_t n_streams, int64_t syms_per_stream,
                              int32_t chunk_syms, int32_t syms_per_pos,
                              int32_t streams_per_session, const uint8_t *bits, int32_t n_tables,
                              const uint16_t *freq, uint32_t *states, uint16_t *words,
                              const uint64_t *word_off, uint64_t word_cap_per_unit,
                              uint32_t *n_words);

int plco_rans_decode_bucketed(const uint16_t *freq, const uint32_t *states, const uint16_t *words,
                              const uint64_t *word_off, const uint32_t *n_words,
                              int64_t n_streams, int64_t syms_per_stream, int32_t chunk_syms,
                              int32_t syms_per_pos, int32_t streams_per_session,
                              const uint8_t *bits, int32_t n_tables, uint8_t *symbols);

#ifdef __cplusplus
}
#endif
#endif
