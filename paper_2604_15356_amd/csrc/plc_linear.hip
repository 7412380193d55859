// Linear-embedding predictor (Sec. 7.1, "Linear embedding approximation"): the KV vector of a layer is
// taken as linear in the embedding of the next token, F(t_<i, t) ~ c(t_<i) + A E(t), so the predicted
// KV vector is  c + A Ebar_i  with  Ebar_i = sum_t P(t | t_<i) E(t)  the expected embedding -- one
// weighted sum over the whole vocabulary.  Both steps are dense contractions and run on the matrix
// cores; see include/plc.h for shapes and layouts.
//
//   expected embedding   Ebar [rows, m]     = P [rows, V] * Et [m, V]^T                (K = V)
//   prediction           pred [n, 2 H d]    = Ebar[s] [n, m] * A[l] [2 H d, m]^T + c   (K = m), per (s, l),
//                        fused with the residual / quantiser (encode) or the add-back (decode).
//
// One kernel: C[M, N] = X[M, K] * Y[N, K]^T, fp16 operands with K contiguous in both, fp32 accumulation
// in v_mfma_f32_32x32x16_f16.  A workgroup of four wavefronts owns a 128 x 128 tile of C, each wavefront
// a 64 x 64 quarter (2 x 2 MFMA tiles, 64 accumulator registers).  K advances in slices of 32 through two
// LDS buffers; the next slice travels global -> registers while the current one is multiplied, and is
// written to the other buffer afterwards, so one barrier per slice suffices.  The 16-byte pieces of a
// slice row are stored swizzled so that the fragment reads of consecutive rows spread over the banks.
#include "plc_device.h"

namespace plc {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int kTileM = 128, kTileN = 128, kTileK = 32;
constexpr int kLdsRow = 32;  // halves per LDS row (64 bytes = four 16-byte pieces, stored swizzled)

// A slice row holds four 16-byte pieces; piece g of row r is stored at position g ^ ((r >> 1) & 3), so that
// eight consecutive rows reading the same piece touch eight different 16-byte columns of the 128-byte bank line.
__device__ __forceinline__ int lds_piece(int row, int g) { return row * kLdsRow + ((g ^ ((row >> 1) & 3)) << 3); }

// Fragment layout of v_mfma_f32_32x32x16_f16 (checked on the device): lane l holds A[l % 32][8 (l / 32) + j],
// B[8 (l / 32) + j][l % 32], j = 0..7, and C[8 (i / 4) + 4 (l / 32) + i % 4][l % 32] in accumulator i = 0..15.
template <class Epilogue>
__global__ __launch_bounds__(256) void gemm_nt_kernel(const _Float16 *__restrict__ X, const _Float16 *__restrict__ Y,
                                                      int64_t x_batch_stride, int64_t y_batch_stride, int32_t x_batch_div,
                                                      int32_t y_batch_mod, int K, int tiles_n, Epilogue ep) {
  __shared__ __attribute__((aligned(16))) _Float16 xs[2][kTileM * kLdsRow];
  __shared__ __attribute__((aligned(16))) _Float16 ys[2][kTileN * kLdsRow];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int batch = blockIdx.y;
  const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x - tile_m * tiles_n;
  // batch -> operand: X of batch b is X + (b / x_batch_div) * stride, Y is Y + (b % y_batch_mod) * stride
  const _Float16 *xb = X + (int64_t)(batch / x_batch_div) * x_batch_stride + (int64_t)tile_m * kTileM * K;
  const _Float16 *yb = Y + (int64_t)(batch % y_batch_mod) * y_batch_stride + (int64_t)tile_n * kTileN * K;

  // global -> LDS: a slice of a tile is 128 rows x 64 bytes = 512 pieces of 16 bytes, two per thread
  const int lrow = threadIdx.x >> 2, lk = (threadIdx.x & 3) * 8;
  const _Float16 *xg = xb + (int64_t)lrow * K + lk;
  const _Float16 *yg = yb + (int64_t)lrow * K + lk;
  const int64_t half_tile = (int64_t)64 * K;
  // Two register sets (A, B) carry the slices two and three steps ahead, so that a global load has two
  // multiply phases to arrive in before it is written to LDS.  (Plain variables and macros, not arrays
  // captured by a lambda: those would live in scratch memory.)
  uint4 ax0, ax1, ay0, ay1, bx0, bx1, by0, by1;
#define PLC_FETCH(R, k0)                                               \
  R##x0 = *reinterpret_cast<const uint4 *>(xg + (k0));                 \
  R##x1 = *reinterpret_cast<const uint4 *>(xg + (k0) + half_tile);     \
  R##y0 = *reinterpret_cast<const uint4 *>(yg + (k0));                 \
  R##y1 = *reinterpret_cast<const uint4 *>(yg + (k0) + half_tile)
#define PLC_LAND(R, buf)                                                           \
  *reinterpret_cast<uint4 *>(&xs[buf][lds_piece(lrow, lk >> 3)]) = R##x0;          \
  *reinterpret_cast<uint4 *>(&xs[buf][lds_piece(lrow + 64, lk >> 3)]) = R##x1;     \
  *reinterpret_cast<uint4 *>(&ys[buf][lds_piece(lrow, lk >> 3)]) = R##y0;          \
  *reinterpret_cast<uint4 *>(&ys[buf][lds_piece(lrow + 64, lk >> 3)]) = R##y1

  float16v acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

  const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
  const int slices = K / kTileK;
  auto multiply = [&](int buf) {
#pragma unroll
    for (int ks = 0; ks < kTileK / 16; ++ks) {
      half8 fa[2], fb[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        fa[t] = *reinterpret_cast<const half8 *>(&xs[buf][lds_piece(wm * 64 + t * 32 + frag_row, (frag_k >> 3) + 2 * ks)]);
        fb[t] = *reinterpret_cast<const half8 *>(&ys[buf][lds_piece(wn * 64 + t * 32 + frag_row, (frag_k >> 3) + 2 * ks)]);
      }
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[a], fb[b], acc[a][b], 0, 0, 0);
    }
  };

  PLC_FETCH(a, 0);
  PLC_LAND(a, 0);
  if (slices > 1) {
    PLC_FETCH(a, kTileK);
  }
  if (slices > 2) {
    PLC_FETCH(b, 2 * kTileK);
  }
  __syncthreads();
  for (int s = 0; s < slices; s += 2) {
    // slice s sits in buffer 0, slice s + 1 in set A, slice s + 2 in set B
    multiply(0);
    if (s + 1 < slices) {
      PLC_LAND(a, 1);
      if (s + 3 < slices) {
        PLC_FETCH(a, (s + 3) * kTileK);
      }
    }
    __syncthreads();
    if (s + 1 < slices) multiply(1);
    if (s + 2 < slices) {
      PLC_LAND(b, 0);
      if (s + 4 < slices) {
        PLC_FETCH(b, (s + 4) * kTileK);
      }
    }
    __syncthreads();
  }
#undef PLC_FETCH
#undef PLC_LAND

  const int row0 = tile_m * kTileM + wm * 64 + 4 * (lane >> 5);
  const int col0 = tile_n * kTileN + wn * 64 + (lane & 31);
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) ep(batch, row0 + a * 32 + 8 * (i >> 2) + (i & 3), col0 + b * 32, acc[a][b][i]);
}

// ---- epilogues --------------------------------------------------------------------------------

struct StoreHalf {  // Ebar[row, col] = fp16(acc)
  _Float16 *out;
  int64_t ld;
  __device__ void operator()(int, int row, int col, float v) const { out[(int64_t)row * ld + col] = (_Float16)v; }
};

struct LinearCoord {
  int32_t L, H, n, d;
  int64_t as[4];
  // batch = s * L + l; col = (h * 2 + c) * d + e
  __device__ void locate(int batch, int row, int col, int *c, int64_t *act_off, int64_t *sym_off) const {
    const int s = batch / L, l = batch - s * L;
    const int hc = col / d, e = col - hc * d;
    const int h = hc >> 1;
    *c = hc & 1;
    *act_off = s * as[0] + l * as[1] + h * as[2] + (int64_t)row * as[3] + e;
    *sym_off = ((((int64_t)batch * H + h) * n + row) * 2 + *c) * d + e;
  }
};

struct EncodeLinear {  // residual against c + A Ebar, quantised (escapes are gathered by a later pass)
  LinearCoord g;
  const _Float16 *bias_k, *bias_v, *act_k, *act_v;
  uint8_t *symbols;
  float delta, qmax;
  __device__ void operator()(int batch, int row, int col, float v) const {
    int c;
    int64_t ao, so;
    g.locate(batch, row, col, &c, &ao, &so);
    const float pred = v + (float)(c ? bias_v : bias_k)[ao];
    const float r = (float)(c ? act_v : act_k)[ao] - pred;
    const float u = r / delta;
    const float qf = __builtin_rintf(u);
    symbols[so] = __builtin_fabsf(qf) <= qmax ? (uint8_t)((int)qf + (int)kZeroSymbol) : (uint8_t)PLC_ESCAPE;
  }
};

struct DecodeLinear {  // c + A Ebar plus the dequantised residual (escaped components are patched by a later pass)
  LinearCoord g;
  const _Float16 *bias_k, *bias_v;
  _Float16 *out_k, *out_v;
  const uint8_t *symbols;
  float delta;
  __device__ void operator()(int batch, int row, int col, float v) const {
    int c;
    int64_t ao, so;
    g.locate(batch, row, col, &c, &ao, &so);
    const float pred = v + (float)(c ? bias_v : bias_k)[ao];
    const float qf = (float)((int)symbols[so] - (int)kZeroSymbol);
    float x = __builtin_fmaf(qf, delta, pred);
    asm("" : "+v"(x));  // round to fp32, then to fp16
    (c ? out_v : out_k)[ao] = (_Float16)x;
  }
};

bool aligned16(const void *p) { return p && (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool linear_shapes_ok(const plc_dims *dm, int32_t m) {
  if (!dm || dm->S < 1 || dm->L < 1 || dm->H < 1) return false;
  if (dm->n < kTileM || dm->n % kTileM) return false;                    // positions: whole tiles of rows
  if (dm->d < 8 || dm->d % 8 || (2 * dm->H * dm->d) % kTileN) return false;  // (head, K/V, component): whole tiles
  if (m < kTileK || m % kTileK) return false;
  if (!(dm->delta > 0.0f) || !(dm->delta < 3.0e38f) || dm->qmax < 1 || dm->qmax > 127) return false;
  for (int a = 0; a < 4; ++a)
    if (dm->act_stride[a] < 0 || dm->act_stride[a] % kChunk) return false;
  return (int64_t)dm->S * dm->L < 65536;  // grid.y
}

LinearCoord coord_of(const plc_dims *dm) {
  LinearCoord g;
  g.L = dm->L;
  g.H = dm->H;
  g.n = dm->n;
  g.d = dm->d;
  for (int i = 0; i < 4; ++i) g.as[i] = dm->act_stride[i];
  return g;
}

}  // namespace
}  // namespace plc

using namespace plc;

extern "C" int plc_expected_embedding(const void *probs_full, const void *embed_t, int64_t rows, int32_t V, int32_t m,
                                      void *ebar, void *stream) {
  if (!aligned16(probs_full) || !aligned16(embed_t) || !aligned16(ebar)) return PLC_ERR_INVALID;
  if (rows < kTileM || rows % kTileM || m < kTileN || m % kTileN || V < kTileK || V % kTileK) return PLC_ERR_INVALID;
  const int64_t tiles = (rows / kTileM) * (m / kTileN);
  if (tiles >= (1ll << 31)) return PLC_ERR_INVALID;
  StoreHalf ep{static_cast<_Float16 *>(ebar), m};
  hipStream_t st = static_cast<hipStream_t>(stream);
  {
    TraceScope trace(PLC_TRACE_EXPECTED_EMBEDDING, st);
    hipLaunchKernelGGL(gemm_nt_kernel<StoreHalf>, dim3((unsigned)tiles, 1), dim3(256), 0, st,
                       static_cast<const _Float16 *>(probs_full), static_cast<const _Float16 *>(embed_t), (int64_t)0,
                       (int64_t)0, 1, 1, V, m / kTileN, ep);
  }
  return launch_status();
}

extern "C" int plc_predict_residual_linear(const plc_dims *dims, const void *ebar, int32_t m, const void *A,
                                           const void *bias_k, const void *bias_v, const void *act_k,
                                           const void *act_v, uint8_t *symbols, uint16_t *esc_vals, uint64_t esc_cap,
                                           uint32_t *esc_cnt, uint64_t *esc_off, void *ws, size_t ws_bytes,
                                           uint32_t *status, void *stream) {
  if (!linear_shapes_ok(dims, m)) return PLC_ERR_INVALID;
  if (!aligned16(ebar) || !aligned16(A) || !aligned16(bias_k) || !aligned16(bias_v) || !aligned16(act_k) ||
      !aligned16(act_v) || !symbols)
    return PLC_ERR_INVALID;
  const int N = 2 * dims->H * dims->d;
  EncodeLinear ep{coord_of(dims),
                  static_cast<const _Float16 *>(bias_k),
                  static_cast<const _Float16 *>(bias_v),
                  static_cast<const _Float16 *>(act_k),
                  static_cast<const _Float16 *>(act_v),
                  symbols,
                  dims->delta,
                  (float)dims->qmax};
  hipStream_t st = static_cast<hipStream_t>(stream);
  {
    TraceScope trace(PLC_TRACE_PREDICT_LINEAR, st);
    hipLaunchKernelGGL(gemm_nt_kernel<EncodeLinear>, dim3((unsigned)((dims->n / kTileM) * (N / kTileN)), dims->S * dims->L),
                       dim3(256), 0, st, static_cast<const _Float16 *>(ebar), static_cast<const _Float16 *>(A),
                       (int64_t)dims->n * m, (int64_t)N * m, dims->L, dims->L, m, N / kTileN, ep);
  }
  if (hipGetLastError() != hipSuccess) return PLC_ERR_HIP;
  return gather_escapes(dims, act_k, act_v, symbols, esc_vals, esc_cap, esc_cnt, esc_off, ws, ws_bytes, status, st);
}

extern "C" int plc_reconstruct_linear(const plc_dims *dims, const void *ebar, int32_t m, const void *A,
                                      const void *bias_k, const void *bias_v, const uint8_t *symbols,
                                      const uint16_t *esc_vals, uint64_t esc_len, const uint64_t *esc_off, void *out_k,
                                      void *out_v, void *ws, size_t ws_bytes, uint32_t *status, void *stream) {
  if (!linear_shapes_ok(dims, m)) return PLC_ERR_INVALID;
  if (!aligned16(ebar) || !aligned16(A) || !aligned16(bias_k) || !aligned16(bias_v) || !aligned16(out_k) ||
      !aligned16(out_v) || !symbols)
    return PLC_ERR_INVALID;
  const int N = 2 * dims->H * dims->d;
  DecodeLinear ep{coord_of(dims),
                  static_cast<const _Float16 *>(bias_k),
                  static_cast<const _Float16 *>(bias_v),
                  static_cast<_Float16 *>(out_k),
                  static_cast<_Float16 *>(out_v),
                  symbols,
                  dims->delta};
  hipStream_t st = static_cast<hipStream_t>(stream);
  {
    TraceScope trace(PLC_TRACE_RECONSTRUCT_LINEAR, st);
    hipLaunchKernelGGL(gemm_nt_kernel<DecodeLinear>, dim3((unsigned)((dims->n / kTileM) * (N / kTileN)), dims->S * dims->L),
                       dim3(256), 0, st, static_cast<const _Float16 *>(ebar), static_cast<const _Float16 *>(A),
                       (int64_t)dims->n * m, (int64_t)N * m, dims->L, dims->L, m, N / kTileN, ep);
  }
  if (hipGetLastError() != hipSuccess) return PLC_ERR_HIP;
  return patch_escapes(dims, symbols, esc_vals, esc_len, esc_off, out_k, out_v, ws, ws_bytes, status, st);
}
