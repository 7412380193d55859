/*
 * plc.h -- predictive delta coding of a transformer KV cache on AMD MI355X
 * (gfx950): the C boundary of libplc.so.
 *
 * The method (paper "Sequential KV Cache Compression via Probabilistic
 * Language Tries", Layer 2): before a KV vector is written to the cache, the
 * model's own next-token distribution predicts it; only the residual is
 * quantised and entropy coded.  Before it is read, the residual is decoded
 * and the identically recomputed prediction is added back (Sec. 7.2,
 * "Integration with the inference loop").
 *
 * Conventions for every entry point
 *   - Plain C ABI.  All data pointers are DEVICE pointers unless a parameter is
 *     marked "host".  `stream` is a hipStream_t passed as void* (NULL = the
 *     default stream).  Calls only enqueue kernels on `stream` and return; they
 *     never synchronise, allocate or free.
 *   - The caller owns every buffer.  `const` inputs are never written.
 *     Scratch comes from a caller-provided workspace (plc_workspace_bytes).
 *   - Return value: PLC_OK, or an error detected on the host before anything
 *     was enqueued (PLC_ERR_INVALID), or a HIP launch failure (PLC_ERR_HIP).
 *   - Errors that depend on the data are reported through `status`, a device
 *     uint32_t the caller zeroes beforehand and reads after synchronising:
 *     kernels raise it (atomic max) to one of the PLC_ERR_* codes.  Outputs of
 *     a call whose status is non-zero are unspecified but every access stays
 *     inside the buffers described here.
 *   - Calls on different streams are independent as long as their buffers
 *     (including workspace and status) are distinct.
 *
 * Data layout
 *   stream   one per (session s, layer l, KV head h): id = (s*L + l)*H + h.
 *   symbol   one byte per KV component.  Inside a stream, component e of
 *            position i sits at t = (i*2 + c)*d + e with c = 0 for K and 1 for
 *            V, so a stream has N = 2*n*d symbols and `symbols` is the
 *            contiguous array u8 [S,L,H,n,2,d].  Symbol q+127 stands for the
 *            quantised residual q in [-qmax, qmax]; 255 is the escape symbol.
 *   escapes  raw fp16 bit patterns of the escaped components, stream after
 *            stream, in symbol order inside each stream.
 *   table    256 x u16 frequencies per stream summing to 4096.
 *   rANS     32 interleaved lanes per coded unit; symbol t belongs to lane
 *            t mod 32; 32-bit states in [2^16, 2^32); 16-bit words.  The
 *            encoder walks symbols last to first and appends words as they are
 *            produced; the decoder walks first to last and consumes the word
 *            list from its end.  A unit is a whole stream (chunk_syms = 0) or a
 *            run of chunk_syms symbols of it (chunk_syms a multiple of 32);
 *            unit id = stream * units_per_stream + chunk.
 */
#ifndef PLC_H
#define PLC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PLC_OK 0
#define PLC_ERR_INVALID 1  /* bad argument, or an invalid probability row / empty histogram  */
#define PLC_ERR_CAPACITY 2 /* an output list (escapes, rANS words) was too small             */
#define PLC_ERR_CORRUPT 3  /* decoder integrity check failed                                 */
#define PLC_ERR_HIP 4      /* the HIP runtime refused a launch                               */

#define PLC_ERR_SCRATCH 5  /* the shape needs more scratch than the library's own buffer has  */

#define PLC_ESCAPE 255     /* escape symbol                                                  */
#define PLC_RANS_LANES 32
#define PLC_RANS_SCALE 4096

typedef struct plc_dims {
  int32_t S, L, H, n, k, d; /* sessions, layers, KV heads, positions, candidates (1..32), head dim (multiple of 8) */
  int64_t cand_stride[5];   /* element strides of the candidate tensors for (s, l, h, i, j); component e is
                               contiguous.  Every stride must be a multiple of 8 (16-byte rows).             */
  int64_t act_stride[4];    /* element strides of actual / reconstructed KV for (s, l, h, i); multiples of 8 */
  float delta;              /* quantiser step, > 0.  The step IS this fp32 value.                            */
  int32_t qmax;             /* largest |q| with a symbol of its own, 1..127                                  */
} plc_dims;

/* Library version: major*10000 + minor*100 + patch. */
int plc_version(void);

/* Static text for a PLC_* code (host pointer, never NULL). */
const char *plc_strerror(int code);

/* Bytes of device workspace plc_predict_residual / plc_reconstruct need for
 * these dimensions (0 if dims are invalid).  Host call. */
size_t plc_workspace_bytes(const plc_dims *dims /* host */);

/* Number of rANS units per stream for a chunk length (1 when chunk_syms = 0). Host call. */
int64_t plc_units_per_stream(int64_t syms_per_stream, int32_t chunk_syms);

/*
 * Encode side, floating-point part.  For every (s,l,h,i) and for K and V:
 *   weights     w_j = p_j / sum_m p_m over the k candidates (Sec. 7.1, "Top-k
 *               approximation": the prediction is renormalised over the top k);
 *   prediction  pred = sum_j w_j * cand_j, accumulated in fp32 with fused
 *               multiply-add, j ascending from 0 (Def. "Predicted KV vector"
 *               restricted to the top k);
 *   residual    r = act - pred (Def. "KV residual");
 *   quantise    q = round-half-even(r / delta) (Sec. 7.2, point 1: the residual
 *               is what gets quantised and stored); symbol q+127 if |q| <= qmax and r/delta is
 *               finite, else 255 with the raw fp16 of `act` appended to the
 *               stream's escape list.
 * One probability row serves every layer, head, K and V of a position.
 *
 *   dims      host; validated (PLC_ERR_INVALID).
 *   cand_k/v  fp16, logical [S,L,H,n,k,d] addressed through dims->cand_stride; 16-byte aligned.
 *   probs     fp32 [S,n,k] contiguous, raw top-k probabilities.  A row with a negative or NaN
 *             entry, or whose sum is not positive and finite, raises status PLC_ERR_INVALID.
 *   act_k/v   fp16, logical [S,L,H,n,d] through dims->act_stride; 16-byte aligned.
 *   symbols   out, u8 [S,L,H,n,2,d] contiguous; 8-byte aligned.
 *   esc_vals  out, u16[esc_cap].  If the escapes do not fit, status PLC_ERR_CAPACITY is raised
 *             and only the first esc_cap entries are written.
 *   esc_cnt   out, u32 [S*L*H]: escapes per stream.
 *   esc_off   out, u64 [S*L*H]: start of each stream's list in esc_vals (exclusive prefix sum).
 *   pred_out  out, nullable: fp32 [S,L,H,n,2,d], the prediction (for inspection and tests).
 *   ws        workspace of at least plc_workspace_bytes(dims) bytes, 256-byte aligned.
 *   status    device u32, see above.
 */
int plc_predict_residual(const plc_dims *dims, const void *cand_k, const void *cand_v,
                         const float *probs, const void *act_k, const void *act_v,
                         uint8_t *symbols, uint16_t *esc_vals, uint64_t esc_cap,
                         uint32_t *esc_cnt, uint64_t *esc_off, float *pred_out,
                         void *ws, size_t ws_bytes, uint32_t *status, void *stream);

/*
 * plc_predict_residual and plc_histogram in one pass: the same outputs as plc_predict_residual, plus
 *   counts   out, u32 [S*L*H, 256]; overwritten with what plc_histogram would count on `symbols`
 * taken while the symbols are produced (per-workgroup histograms in LDS, added to `counts` with integer
 * atomics: the result does not depend on the order), so that the symbols need not be read back for the
 * statistics.  Everything else as in plc_predict_residual.
 */
int plc_predict_residual_hist(const plc_dims *dims, const void *cand_k, const void *cand_v,
                              const float *probs, const void *act_k, const void *act_v,
                              uint8_t *symbols, uint16_t *esc_vals, uint64_t esc_cap,
                              uint32_t *esc_cnt, uint64_t *esc_off, float *pred_out, uint32_t *counts,
                              void *ws, size_t ws_bytes, uint32_t *status, void *stream);

/*
 * plc_predict_residual for callers that cannot allocate device memory or have a workspace handed to
 * them: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels and results, bit for bit, but the workspace is a buffer inside the library itself
 * (a static device array of PLC_STATIC_SCRATCH_BYTES bytes; every GPU the library runs on holds its own
 * copy until the process ends).  The call allocates and frees nothing.
 *   - Shapes with plc_workspace_bytes(dims) > PLC_STATIC_SCRATCH_BYTES are refused with PLC_ERR_SCRATCH
 *     before anything is enqueued (48 MiB covers 1.6e8 KV components per call, e.g. L=32, H=8, d=128,
 *     n=4096).
 *   - The first call on a device looks the buffer's address up (hipGetSymbolAddress with that device
 *     current) and must be made outside stream capture; PLC_ERR_HIP if the lookup fails.
 *   - All calls on one GPU share that GPU's buffer: calls that overlap in time on one GPU (different
 *     streams, or different threads) race.  Calls that follow each other on one stream do not: every part
 *     of the buffer a kernel reads was written earlier in the same call, so nothing carries over from
 *     the call before, whatever its shape.
 */
#define PLC_STATIC_SCRATCH_BYTES (48u << 20)
int plc_predict_residual_noalloc(const plc_dims *dims, const void *cand_k, const void *cand_v,
                                 const float *probs, const void *act_k, const void *act_v,
                                 uint8_t *symbols, uint16_t *esc_vals, uint64_t esc_cap,
                                 uint32_t *esc_cnt, uint64_t *esc_off, float *pred_out,
                                 uint32_t *status, void *stream);

/*
 * Per-stream symbol statistics for the entropy coder (the paper only asks
 * for a source code of the residuals near their entropy, proof of Prop. "Layer
 * orthogonality", Sec. 6.1, and names no coder; statistics, table and
 * bitstream are this library's own format, defined here).
 *   symbols  u8 [n_streams, syms_per_stream] contiguous.
 *   counts   out, u32 [n_streams, 256]; overwritten.  syms_per_stream < 2^32.
 */
int plc_histogram(const uint8_t *symbols, int64_t n_streams, int64_t syms_per_stream,
                  uint32_t *counts, void *stream);

/*
 * Counts -> integer frequency table on the 2^12 scale, integer arithmetic
 * only (the paper is silent on the coder's tables; this normalisation is the
 * format's own).  With C the inclusive running count and T the total,
 *   f[s] = floor(C[s] * 4096 / T) - floor(C[s-1] * 4096 / T);
 * then, for s ascending, every symbol that occurs but got f[s] = 0 takes one
 * unit from the currently largest frequency (lowest symbol on ties).
 *   counts  u32 [n_streams, 256].  A stream with T = 0 raises status PLC_ERR_INVALID.
 *   freq    out, u16 [n_streams, 256]  (a single-symbol stream has f = 4096).
 *   cum     out, nullable: u16 [n_streams, 257], exclusive prefix sums of freq.
 */
int plc_build_freq(const uint32_t *counts, int64_t n_streams, uint16_t *freq, uint16_t *cum,
                   uint32_t *status, void *stream);

/*
 * rANS encoder (the paper fixes no entropy coder, see plc_histogram; every
 * constant and the word order below are the format's own).  For each unit,
 * with x = 2^16 in all 32 lanes initially and
 * for t from the unit's last symbol down to its first (lane = t mod 32):
 *   if (x >> 20) >= f[sym]:  append (x & 0xffff) to the unit's words, x >>= 16
 *   x = (x / f[sym]) * 4096 + (x % f[sym]) + cum[sym]
 *   symbols   u8 [n_streams, syms_per_stream].
 *   freq      u16 [n_streams, 256] summing to 4096 with f > 0 for every symbol that occurs;
 *             a symbol with f = 0 in the data raises status PLC_ERR_INVALID.
 *   states    out, u32 [n_units, 32]: final lane states.
 *   words     out, u16: unit u writes words[word_off[u] .. word_off[u] + n_words[u]).
 *   word_off  u64 [n_units], chosen by the caller; word_cap_per_unit entries are reserved for
 *             each unit.  A unit never needs more words than it has symbols.  If the
 *             reservation is too small, status PLC_ERR_CAPACITY is raised and nothing is
 *             written past it.
 *   n_words   out, u32 [n_units].
 */
int plc_rans_encode(const uint8_t *symbols, int64_t n_streams, int64_t syms_per_stream,
                    int32_t chunk_syms, const uint16_t *freq, uint32_t *states,
                    uint16_t *words, const uint64_t *word_off, uint64_t word_cap_per_unit,
                    uint32_t *n_words, uint32_t *status, void *stream);

/*
 * rANS decoder, the exact inverse (same remark: the format's own definition,
 * not the paper's).  For each unit, x = states, ptr = n_words,
 * and for t from the unit's first symbol to its last (lane = t mod 32):
 *   slot = x & 4095;  sym = the s with cum[s] <= slot < cum[s+1]
 *   x = f[sym] * (x >> 12) + slot - cum[sym]
 *   if x < 2^16:  x = (x << 16) | words[--ptr]
 * At the end ptr must be 0 and every lane state 2^16, otherwise status
 * PLC_ERR_CORRUPT is raised.  Reads stay inside words[0 .. words_len) and
 * inside each unit's [word_off, word_off + n_words) whatever the data holds.
 *   symbols   out, u8 [n_streams, syms_per_stream].
 */
int plc_rans_decode(const uint16_t *freq, const uint32_t *states, const uint16_t *words,
                    uint64_t words_len, const uint64_t *word_off, const uint32_t *n_words,
                    int64_t n_streams, int64_t syms_per_stream, int32_t chunk_syms,
                    uint8_t *symbols, uint32_t *status, void *stream);

/*
 * Decode side, floating-point part (Sec. 7.2, point 2: the stored residual is
 * dequantised and added to a prediction that the reader forms exactly as the
 * writer did; Prop. "Three-layer composition", correctness: the error of the
 * recovered KV is the quantiser's error on the residual).  The prediction is computed exactly as in
 * plc_predict_residual; then x = fma((float)(sym - 127), delta, pred), rounded
 * to fp16 (nearest even).  An escape symbol takes the next raw fp16 of its
 * stream's escape list instead.
 *   symbols   u8 [S,L,H,n,2,d].
 *   esc_vals  u16[esc_len]; esc_off u64 [S*L*H] as produced by plc_predict_residual.  An escape
 *             whose list index falls outside esc_len raises status PLC_ERR_CORRUPT.
 *   out_k/v   out, fp16 logical [S,L,H,n,d] through dims->act_stride; 16-byte aligned.
 */
int plc_reconstruct(const plc_dims *dims, const void *cand_k, const void *cand_v,
                    const float *probs, const uint8_t *symbols, const uint16_t *esc_vals,
                    uint64_t esc_len, const uint64_t *esc_off, void *out_k, void *out_v,
                    void *ws, size_t ws_bytes, uint32_t *status, void *stream);

/*
 * plc_rans_decode followed by plc_reconstruct, as one call (the decode side of
 * Sec. 7.2 as a whole: entropy-decode the residual symbols, dequantise, add back
 * the prediction).  Results -- symbols, out_k, out_v, status -- are those of the
 * two calls, bit for bit.  With one rANS unit per stream (chunk_syms = 0) and
 * k <= 8 the reconstruction runs inside the entropy decoder: a unit's symbols
 * come out in stream order, so a further wavefront of the unit's workgroup
 * turns each batch of them into KV components while the next batch is being
 * decoded, with the candidates it needs requested ahead of time and the
 * escaped components taken from the escape lists.  For every other shape the
 * call simply makes the two calls.
 * Arguments as in plc_rans_decode (n_streams = S*L*H and syms_per_stream =
 * 2*n*d follow from dims) and plc_reconstruct; symbols is an output here.
 */
int plc_rans_decode_reconstruct(const plc_dims *dims, const uint16_t *freq, const uint32_t *states,
                                const uint16_t *words, uint64_t words_len, const uint64_t *word_off,
                                const uint32_t *n_words, int32_t chunk_syms, const void *cand_k,
                                const void *cand_v, const float *probs, const uint16_t *esc_vals,
                                uint64_t esc_len, const uint64_t *esc_off, uint8_t *symbols,
                                void *out_k, void *out_v, void *ws, size_t ws_bytes,
                                uint32_t *status, void *stream);

/*
 * ---- Token-conditional coding -------------------------------------------------
 * Lemma "KV determinism" (Sec. 4.1): the KV vector of a position is a function
 * of the token prefix.  So when the token that was actually produced is one of
 * the k candidates, its candidate vector IS the prediction, the residual is
 * only what numerical noise separates the two, and all that has to be stored
 * besides is which candidate it was -- at a cost of the token's surprisal
 * (Thm. "Sequential entropy bound", Sec. 4.2).  The calls below add that path
 * next to the weighted-mean path above; histogram, table and rANS calls serve
 * both.
 *
 *   chosen   i32 [S,n], one entry per (session, position), shared by every
 *            layer, head, K and V:  j in [0,k) = the token is candidate j, the
 *            prediction is cand_j itself (its fp16 values, exactly);  -1 = the
 *            token is not among the candidates, the prediction is the weighted
 *            mean exactly as in plc_predict_residual.  Any other value raises
 *            status PLC_ERR_INVALID and is treated as -1.
 * Everything else (arguments, layouts, escapes, workspace, status) is as in
 * the call of the same name without the suffix.
 */
int plc_predict_residual_cond(const plc_dims *dims, const void *cand_k, const void *cand_v,
                              const float *probs, const int32_t *chosen, const void *act_k,
                              const void *act_v, uint8_t *symbols, uint16_t *esc_vals,
                              uint64_t esc_cap, uint32_t *esc_cnt, uint64_t *esc_off,
                              float *pred_out, void *ws, size_t ws_bytes, uint32_t *status,
                              void *stream);

int plc_reconstruct_cond(const plc_dims *dims, const void *cand_k, const void *cand_v,
                         const float *probs, const int32_t *chosen, const uint8_t *symbols,
                         const uint16_t *esc_vals, uint64_t esc_len, const uint64_t *esc_off,
                         void *out_k, void *out_v, void *ws, size_t ws_bytes, uint32_t *status,
                         void *stream);

/* plc_rans_decode followed by plc_reconstruct_cond as one call, the way
 * plc_rans_decode_reconstruct stands for plc_rans_decode and plc_reconstruct:
 * same results, and under the same conditions -- here also: with more than
 * four candidates at most 2048 streams, beyond which the two calls are the
 * faster -- one kernel, whose
 * reconstructing wavefront fetches each position's chosen index a round before
 * it requests that candidate (all k of them where a position has none).
 * chosen must be in place on `stream` (plc_index_decode) before the call. */
int plc_rans_decode_reconstruct_cond(const plc_dims *dims, const uint16_t *freq,
                                     const uint32_t *states, const uint16_t *words,
                                     uint64_t words_len, const uint64_t *word_off,
                                     const uint32_t *n_words, int32_t chunk_syms,
                                     const void *cand_k, const void *cand_v, const float *probs,
                                     const int32_t *chosen, const uint16_t *esc_vals,
                                     uint64_t esc_len, const uint64_t *esc_off, uint8_t *symbols,
                                     void *out_k, void *out_v, void *ws, size_t ws_bytes,
                                     uint32_t *status, void *stream);

/*
 * `chosen` from the vectors alone, for an encoder that is not told the token:
 * by the same lemma one row identifies it.  Per (s, i): D_j = sum_e (act[e] -
 * cand_j[e])^2 over the key row of layer 0, head 0 (fp32; the difference, then
 * a fused multiply-add accumulate, e ascending); chosen = the j with the
 * smallest D_j (lowest j on ties; a NaN distance never wins), or -1 when that
 * distance exceeds max_mean_sq * d or no distance compares.
 *   cand_k, act_k  as in plc_predict_residual.   chosen  out, i32 [S,n].
 */
int plc_select_candidate(const plc_dims *dims, const void *cand_k, const void *act_k,
                         float max_mean_sq, int32_t *chosen, void *stream);

/*
 * The index stream: `chosen` coded under the model's own probabilities, one
 * 32-lane rANS unit per session (same coder as plc_rans_encode: position i in
 * lane i mod 32, last position first, 16-bit words in emission order), with a
 * table per position.  Position (s,i) has k+1 symbols, j < k for chosen = j
 * and k for chosen = -1, with frequencies on the 2^12 scale made from the raw
 * probabilities p = probs[s,i,:] in fp32:  c_0 = 0, c_{j+1} = c_j + p_j;
 * b_j = min(4096, floor(4096 * c_j)) for j <= k, b_{k+1} = 4096;  f_j =
 * b_{j+1} - b_j;  then, j ascending, every f_j = 0 takes one unit from the
 * currently largest frequency (lowest index on ties).  The symbol k so owns
 * the probability the top k leave, and a chosen candidate costs about
 * -log2 p_j bits.  A row with a negative or NaN entry raises status
 * PLC_ERR_INVALID (its bad entries count as 0).
 *   probs     fp32 [S,n,k].   chosen  i32 [S,n] (values outside [-1,k): PLC_ERR_INVALID, coded as -1).
 *   states    out, u32 [S,32].   words  out, u16: session s writes words[word_off[s] .. + n_words[s]);
 *   word_cap  entries reserved per session (n always suffices); overflow raises PLC_ERR_CAPACITY
 *             and nothing is written past the reservation.   n_words  out, u32 [S].
 */
int plc_index_encode(const float *probs, const int32_t *chosen, int32_t S, int32_t n, int32_t k,
                     uint32_t *states, uint16_t *words, const uint64_t *word_off,
                     uint64_t word_cap, uint32_t *n_words, uint32_t *status, void *stream);

/* Inverse of plc_index_encode; same integrity rule as plc_rans_decode (all words used, all
 * lanes back at 2^16, else PLC_ERR_CORRUPT); reads stay inside words[0 .. words_len).
 *   chosen  out, i32 [S,n]. */
int plc_index_decode(const float *probs, const uint32_t *states, const uint16_t *words,
                     uint64_t words_len, const uint64_t *word_off, const uint32_t *n_words,
                     int32_t S, int32_t n, int32_t k, int32_t *chosen, uint32_t *status,
                     void *stream);

/*
 * ---- Surprisal-adaptive quantiser ---------------------------------------------
 * Def. "Surprisal-adaptive quantizer" (Sec. 5.3): position i gets b_i = max(1,
 * floor(b0 * h_i / hbar)) bits per residual component, h_i its surprisal and
 * hbar the average; Cor. "Practical bit allocation" (Sec. 9.4): b bits stand
 * for a uniform step of range / 2^b.  Here b_i is capped at PLC_MAX_BITS, the
 * step of position i is the fp32 value range * 2^-b_i (an exact scaling), and
 * the symbols of positions with depth b are counted and coded with table number
 * b - 1 of their stream, so that each depth has statistics of its own.
 *
 *   bits    u8 [S,n], values 1..PLC_MAX_BITS, shared by all layers, heads, K and V of a position
 *           (any other value raises status PLC_ERR_INVALID and counts as 1).
 *   range   fp32 > 0.
 */
#define PLC_MAX_BITS 4

/*
 * b_i from the token's coded surprisal h_i = log2(4096 / f), f the frequency of the position's
 * index symbol (see plc_index_encode; symbol k for chosen = -1):
 *   floor(b0 * h_i / hbar) >= m   <=>   f <= 4096 * 2^(-m * hbar / b0),
 * so with thr[m] = floor(4096 * 2^(-m * hbar / b0)) for m = 2..bmax (host array of bmax + 1
 * entries, entries 0 and 1 unused, non-increasing) the depth is the largest m with f <= thr[m],
 * or 1.  Integer comparisons only: encoder and decoder agree bit for bit.
 *   bits  out, u8 [S,n].
 */
/* The thresholds of that comparison from the definition's two parameters (Def. "Surprisal-adaptive
 * quantizer", Sec. 5.3: b0 the base depth, hbar the average surprisal in bits): thr[m] =
 * floor(4096 * 2^(-m * hbar / b0)) in double precision for m = 2..bmax, thr[0] = thr[1] = 0.  Host call;
 * thr is a HOST array of bmax + 1 entries.  PLC_ERR_INVALID unless b0, hbar > 0 and finite and
 * 1 <= bmax <= PLC_MAX_BITS (the definition puts no upper limit on b_i; this library codes at most
 * PLC_MAX_BITS depths and refuses more). */
int plc_surprisal_thresholds(double b0, double hbar, int32_t bmax, uint16_t *thr /* host */);

int plc_surprisal_bits(const float *probs, const int32_t *chosen, int32_t S, int32_t n, int32_t k,
                       const uint16_t *thr /* host */, int32_t bmax, uint8_t *bits,
                       uint32_t *status, void *stream);

/* As plc_predict_residual_cond / plc_reconstruct_cond (chosen all -1 = weighted mean everywhere),
 * with the step of position (s,i) = range * 2^-bits[s,i] in place of dims->delta. */
int plc_predict_residual_adapt(const plc_dims *dims, const void *cand_k, const void *cand_v,
                               const float *probs, const int32_t *chosen, const uint8_t *bits,
                               float range, const void *act_k, const void *act_v, uint8_t *symbols,
                               uint16_t *esc_vals, uint64_t esc_cap, uint32_t *esc_cnt,
                               uint64_t *esc_off, float *pred_out, void *ws, size_t ws_bytes,
                               uint32_t *status, void *stream);

int plc_reconstruct_adapt(const plc_dims *dims, const void *cand_k, const void *cand_v,
                          const float *probs, const int32_t *chosen, const uint8_t *bits,
                          float range, const uint8_t *symbols, const uint16_t *esc_vals,
                          uint64_t esc_len, const uint64_t *esc_off, void *out_k, void *out_v,
                          void *ws, size_t ws_bytes, uint32_t *status, void *stream);

/*
 * Statistics, tables and rANS with one table per depth.  Stream st belongs to session
 * st / streams_per_session; symbol t of a stream belongs to position t / syms_per_pos
 * (syms_per_pos = 2d for the KV layout; a multiple of 32, so that a group of 32 symbols never
 * straddles two positions; syms_per_stream a multiple of it).
 *   counts  out, u32 [n_streams, n_tables, 256];   freq  u16 [n_streams, n_tables, 256]: a depth that
 *           does not occur in a stream has an all-zero table, the others sum to 4096 exactly as in
 *           plc_build_freq.  n_tables in 1..PLC_MAX_BITS.  symbols 16-byte aligned.
 * Everything else as in plc_histogram / plc_build_freq / plc_rans_encode / plc_rans_decode.
 */
int plc_histogram_bucketed(const uint8_t *symbols, int64_t n_streams, int64_t syms_per_stream,
                           int32_t syms_per_pos, int32_t streams_per_session, const uint8_t *bits,
                           int32_t n_tables, uint32_t *counts, uint32_t *status, void *stream);

int plc_build_freq_bucketed(const uint32_t *counts, int64_t n_streams, int32_t n_tables,
                            uint16_t *freq, uint32_t *status, void *stream);

int plc_rans_encode_bucketed(const uint8_t *symbols, int64_t n_streams, int64_t syms_per_stream,
                             int32_t chunk_syms, int32_t syms_per_pos, int32_t streams_per_session,
                             const uint8_t *bits, int32_t n_tables, const uint16_t *freq,
                             uint32_t *states, uint16_t *words, const uint64_t *word_off,
                             uint64_t word_cap_per_unit, uint32_t *n_words, uint32_t *status,
                             void *stream);

int plc_rans_decode_bucketed(const uint16_t *freq, const uint32_t *states, const uint16_t *words,
                             uint64_t words_len, const uint64_t *word_off, const uint32_t *n_words,
                             int64_t n_streams, int64_t syms_per_stream, int32_t chunk_syms,
                             int32_t syms_per_pos, int32_t streams_per_session, const uint8_t *bits,
                             int32_t n_tables, uint8_t *symbols, uint32_t *status, void *stream);

/* plc_rans_decode_bucketed (syms_per_pos = 2d, streams_per_session = L*H) followed by
 * plc_reconstruct_adapt as one call, the way plc_rans_decode_reconstruct stands for
 * plc_rans_decode and plc_reconstruct: same results, and under the same conditions (here also: at
 * most 512 streams) one kernel, whose reconstructing wavefront fetches each position's depth with
 * its chosen index.  chosen and bits must be in place on `stream` before the call. */
int plc_rans_decode_reconstruct_adapt(const plc_dims *dims, const uint16_t *freq,
                                      const uint32_t *states, const uint16_t *words,
                                      uint64_t words_len, const uint64_t *word_off,
                                      const uint32_t *n_words, int32_t chunk_syms, int32_t n_tables,
                                      const void *cand_k, const void *cand_v, const float *probs,
                                      const int32_t *chosen, const uint8_t *bits, float range,
                                      const uint16_t *esc_vals, uint64_t esc_len,
                                      const uint64_t *esc_off, uint8_t *symbols, void *out_k,
                                      void *out_v, void *ws, size_t ws_bytes, uint32_t *status,
                                      void *stream);

/*
 * ---- Linear-embedding predictor ------------------------------------------------
 * Sec. 7.1, "Linear embedding approximation": per layer the KV vector is taken as linear in the
 * embedding of the next token, F(t_<i, t) ~ c(t_<i) + A E(t), so that the predicted KV vector is
 * c + A Ebar_i with Ebar_i = sum_t P(t | t_<i) E(t), the expected embedding -- one weighted sum over
 * the whole vocabulary.  Readings: A is one matrix per layer (a per-position matrix, as the text has
 * it, would outweigh the cache by orders of magnitude); c has the shape of the KV cache.  Both steps
 * are dense contractions (fp16 operands, fp32 accumulation on the matrix cores).
 *
 *   probs_full  fp16 [rows, V], rows = S*n: the full next-token distribution of every position.
 *   embed_t     fp16 [m, V]: the embedding table, transposed (vocabulary index contiguous).
 *   ebar        fp16 [rows, m] (out of plc_expected_embedding, in of the other two).
 *   A           fp16 [L, H, 2, d, m]: row (h, c, e) of layer l maps an embedding to component e of
 *               K (c = 0) or V (c = 1) of head h.
 *   bias_k/v    fp16, logical [S,L,H,n,d] through dims->act_stride (the c of the formula).
 * rows, n multiples of 128; m and 2*H*d multiples of 128; V a multiple of 32; all pointers 16-byte
 * aligned.  dims->k and dims->cand_stride are not used.  Residual, quantiser, symbols, escapes and
 * the reconstruction are those of plc_predict_residual / plc_reconstruct with this prediction; the
 * accumulation order inside the matrix cores is the hardware's, the same on the encode and the
 * decode side.
 */
int plc_expected_embedding(const void *probs_full, const void *embed_t, int64_t rows, int32_t V,
                           int32_t m, void *ebar, void *stream);

int plc_predict_residual_linear(const plc_dims *dims, const void *ebar, int32_t m, const void *A,
                                const void *bias_k, const void *bias_v, const void *act_k,
                                const void *act_v, uint8_t *symbols, uint16_t *esc_vals,
                                uint64_t esc_cap, uint32_t *esc_cnt, uint64_t *esc_off, void *ws,
                                size_t ws_bytes, uint32_t *status, void *stream);

int plc_reconstruct_linear(const plc_dims *dims, const void *ebar, int32_t m, const void *A,
                           const void *bias_k, const void *bias_v, const uint8_t *symbols,
                           const uint16_t *esc_vals, uint64_t esc_len, const uint64_t *esc_off,
                           void *out_k, void *out_v, void *ws, size_t ws_bytes, uint32_t *status,
                           void *stream);

/*
 * ---- Prefix index (host only) ---------------------------------------------------
 * Sec. 7.3, "Trie-Based Prefix Index": the structure in front of this path that finds, for a new
 * session, the stored session whose KV cache it can be coded against: a trie over token sequences
 * with insert, best-match lookup and evict, each linear in the prefix length.  All arguments are
 * HOST pointers; nothing here touches the GPU; a trie is not thread-safe.  Readings: Sec. 7.3 prunes
 * the trie where a node's probability falls under a threshold, taken here as: a prefix is stored only
 * down to the last token at which its surprisal sum stays <= max_bits (= -log2 of that threshold); the
 * best match is the stored prefix with the longest common prefix with the query (the walk down the
 * query's path to the point where no stored path continues, which is the traversal the section gives),
 * for which the trie metric of Def. "PLT trie metric", d_T = -log2 P(common prefix), is returned (the
 * section states the objective once as the largest d_T and once as the most probable common prefix,
 * which contradict each other; the traversal it describes is what is implemented).
 *
 *   tokens  i32 [n];  bits  fp32 [n], nullable: surprisal -log2 P(token | path) of each token, >= 0.
 *   id      caller's handle of a stored prefix, >= 0, unique.
 * plc_trie_insert: *stored_len (nullable) = tokens kept.  PLC_ERR_CAPACITY if another stored prefix
 *   already ends at the same node (the two are indistinguishable to the index); nothing changes then.
 * plc_trie_best_match: *id = a stored prefix sharing the longest common prefix with the query (-1 if
 *   the trie is empty), *lcp = its length in tokens, *dist = sum of `bits` along it.
 * plc_trie_evict: removes a stored prefix and the nodes no stored prefix passes through any more.
 */
typedef struct plc_trie plc_trie;
plc_trie *plc_trie_create(double max_bits);
void plc_trie_destroy(plc_trie *trie);
int64_t plc_trie_size(const plc_trie *trie);  /* stored prefixes */
int64_t plc_trie_nodes(const plc_trie *trie); /* nodes, the root included */
int plc_trie_insert(plc_trie *trie, const int32_t *tokens, const float *bits, int64_t n, int64_t id,
                    int64_t *stored_len);
int plc_trie_best_match(const plc_trie *trie, const int32_t *tokens, int64_t n, int64_t *id,
                        int64_t *lcp, double *dist);
int plc_trie_evict(plc_trie *trie, int64_t id);

/*
 * Instrumentation for benchmarks (not part of the coding path; process-wide,
 * not thread-safe).  While a pair of hipEvent_t (passed as void*) is set for
 * a kernel id, each later call records `start` immediately before and `stop`
 * immediately after that call's main kernel on the call's stream, so that the
 * kernel alone can be timed from outside.  Pass NULLs to clear.  Host call.
 */
#define PLC_TRACE_PREDICT 0     /* main kernel of plc_predict_residual */
#define PLC_TRACE_RECONSTRUCT 1 /* main kernel of plc_reconstruct      */
#define PLC_TRACE_HISTOGRAM 2
#define PLC_TRACE_RANS_ENCODE 3
#define PLC_TRACE_RANS_DECODE 4
#define PLC_TRACE_PREDICT_COND 5     /* main kernel of plc_predict_residual_cond */
#define PLC_TRACE_RECONSTRUCT_COND 6 /* main kernel of plc_reconstruct_cond      */
#define PLC_TRACE_EXPECTED_EMBEDDING 7 /* plc_expected_embedding                     */
#define PLC_TRACE_PREDICT_LINEAR 8     /* contraction of plc_predict_residual_linear */
#define PLC_TRACE_RECONSTRUCT_LINEAR 9 /* contraction of plc_reconstruct_linear      */
#define PLC_TRACE_COUNT 10
int plc_trace_kernel_events(int kernel_id, void *start, void *stop);

#ifdef __cplusplus
}
#endif
#endif /* PLC_H */
