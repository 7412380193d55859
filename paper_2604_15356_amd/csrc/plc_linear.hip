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
// in v_mfma_f32_32x32x16_f16.  A workgroup of WM x WN wavefronts owns a tile of C, each wavefront FM x FN
// MFMA tiles of 32 x 32 of it.  K advances in slices of 64 through two LDS buffers: while slice s is
// multiplied, slice s + 1 moves from registers to the other buffer and slice s + 2 from global memory
// into those registers, one piece at a time between the products; one barrier per slice.
#include "plc_device.h"

namespace plc {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int kTileK = 64;

// LDS layout of one operand slice (R rows x 64 halves): eight pieces of 16 bytes along K, each piece holding
// its R rows back to back (a multiply fragment then reads two runs of 512 contiguous bytes, which the LDS
// serves at its full rate), with 16 bytes of padding between pieces so that the eight pieces of one row,
// written together when the slice lands, fall on different banks.
template <int WM_, int WN_, int FM_, int FN_>
struct GemmShape {
  static constexpr int kWavesM = WM_, kWavesN = WN_, kFragsM = FM_, kFragsN = FN_;
  static constexpr int kWaves = WM_ * WN_, kThreads = 64 * kWaves;
  static constexpr int kTileM = 32 * FM_ * WM_, kTileN = 32 * FN_ * WN_;
  static constexpr int kStrideX = kTileM * 8 + 8, kStrideY = kTileN * 8 + 8;  // halves from piece to piece
  static constexpr int kBufHalves = 8 * (kStrideX + kStrideY);               // both operands, one buffer
  static constexpr size_t kLdsBytes = 2 * kBufHalves * sizeof(_Float16);
  static constexpr int kLandX = kTileM * 8 / kThreads, kLandY = kTileN * 8 / kThreads;  // 16-byte pieces per thread
  static_assert(kLandX * kThreads == kTileM * 8 && kLandY * kThreads == kTileN * 8, "whole pieces per thread");
  static_assert(kTileM % 64 == 0 && kTileN % 64 == 0, "rows land in blocks of 64");
};
using SmallTile = GemmShape<2, 2, 2, 2>;  // 128 x 128, 256 threads, two workgroups per compute unit
using LargeTile = GemmShape<2, 2, 4, 4>;  // 256 x 256, 256 threads, 256 accumulator registers per lane

// Fragment layout of v_mfma_f32_32x32x16_f16 (checked on the device): lane l holds A[l % 32][8 (l / 32) + j],
// B[8 (l / 32) + j][l % 32], j = 0..7, and C[8 (i / 4) + 4 (l / 32) + i % 4][l % 32] in accumulator i = 0..15.
template <class Shape, class Epilogue>
__global__ __launch_bounds__(Shape::kThreads) void gemm_nt_kernel(const _Float16 *__restrict__ X,
                                                                  const _Float16 *__restrict__ Y, int64_t x_batch_stride,
                                                                  int64_t y_batch_stride, int32_t x_batch_div,
                                                                  int32_t y_batch_mod, int K, int tiles_n, Epilogue ep) {
  constexpr int FM = Shape::kFragsM, FN = Shape::kFragsN;
  constexpr int SX = Shape::kStrideX, SY = Shape::kStrideY;
  extern __shared__ __attribute__((aligned(16))) _Float16 gemm_lds[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform: keeps what depends on it in scalar registers
  const int wm = wave / Shape::kWavesN, wn = wave - wm * Shape::kWavesN;
  const int batch = blockIdx.y;
  const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x - tile_m * tiles_n;
  // batch -> operand: X of batch b is X + (b / x_batch_div) * stride, Y is Y + (b % y_batch_mod) * stride
  const _Float16 *xb = X + (int64_t)(batch / x_batch_div) * x_batch_stride + (int64_t)tile_m * Shape::kTileM * K;
  const _Float16 *yb = Y + (int64_t)(batch % y_batch_mod) * y_batch_stride + (int64_t)tile_n * Shape::kTileN * K;

  // global -> LDS: eight consecutive threads fetch one row's 128 bytes of the slice.  The eight rows that one
  // wavefront fetches together lie eight apart, which spreads its LDS writes over all banks: piece i of a
  // thread is row  row_of(i) + 8 j + wave % 8  with j = (thread / 8) % 8, where row_of(i) is the same for the
  // whole workgroup.  A lane that would read past the end of a row re-reads the row's last piece instead.
  const int lp = threadIdx.x & 7, lj = (threadIdx.x >> 3) & 7;
  auto row_of = [](int i, int w) {  // w: wavefront, uniform
    const int q = w + Shape::kWaves * i;
    return 64 * (q >> 3) + (q & 7);
  };
  const int k_mine = lp * 8, k_last = K - 8;
  const unsigned g_lane = (unsigned)(8 * lj) * (unsigned)K;  // halves; tiles stay far below 2^31 halves from xb / yb
  const int l_lane = lj * 64;                                // halves: row 8 j of a piece
  uint4 px[Shape::kLandX], py[Shape::kLandY];
  auto fetch_x = [&](int i, unsigned koff) {
    return *reinterpret_cast<const uint4 *>(xb + (int64_t)row_of(i, wave) * K + (g_lane + koff));
  };
  auto fetch_y = [&](int i, unsigned koff) {
    return *reinterpret_cast<const uint4 *>(yb + (int64_t)row_of(i, wave) * K + (g_lane + koff));
  };

  float16v acc[FM][FN];
#pragma unroll
  for (int a = 0; a < FM; ++a)
#pragma unroll
    for (int b = 0; b < FN; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

  // Fragments: lane l reads row (l % 32) of a 32-row block, K piece 2 ks + l / 32.
  const int frag_x = (lane >> 5) * SX + (wm * FM * 32 + (lane & 31)) * 8;
  const int frag_y = (lane >> 5) * SY + (wn * FN * 32 + (lane & 31)) * 8;
  half8 fa[2][FM], fb[2][FN];

  // Slices: when K is an odd multiple of 32 the first slice is the short one (32 columns, its other half
  // zero in LDS), so that every later slice is whole and the main loop needs no special case.
  const int head = (K & (kTileK - 1)) ? kTileK / 2 : kTileK;
  const int slices = 1 + (K - head) / kTileK;
  {
    _Float16 *const xs = gemm_lds, *const ys = xs + 8 * SX;
    const bool in = k_mine < head;
    const unsigned koff = (unsigned)min(k_mine, k_last);
#pragma unroll
    for (int i = 0; i < Shape::kLandX; ++i) {
      uint4 v = fetch_x(i, koff);
      if (!in) v = make_uint4(0u, 0u, 0u, 0u);
      *reinterpret_cast<uint4 *>(&xs[lp * SX + l_lane + row_of(i, wave) * 8]) = v;
    }
#pragma unroll
    for (int i = 0; i < Shape::kLandY; ++i) {
      uint4 v = fetch_y(i, koff);
      if (!in) v = make_uint4(0u, 0u, 0u, 0u);
      *reinterpret_cast<uint4 *>(&ys[lp * SY + l_lane + row_of(i, wave) * 8]) = v;
    }
    const unsigned koff1 = (unsigned)min(head + k_mine, k_last);  // slice 1 (unused if there is none)
#pragma unroll
    for (int i = 0; i < Shape::kLandX; ++i) px[i] = fetch_x(i, koff1);
#pragma unroll
    for (int i = 0; i < Shape::kLandY; ++i) py[i] = fetch_y(i, koff1);
  }
  __syncthreads();

  // One step per slice: slice s sits in buffer s % 2, slice s + 1 in the registers, and the fragments of
  // the slice's first K step are already loaded.  The step has 4 * FM slots of FN products each; before the
  // products of a slot are issued, the slot requests two fragments of the next K step and, during the first
  // three K steps, writes register pieces of slice s + 1 to the other buffer and refills them from slice
  // s + 2.  Memory instructions are thus spread under the products instead of queueing up in front of them.
  // The barrier stands before the last K step: by then slice s + 1 is complete in LDS and every fragment
  // of slice s has been read, so the last K step can already request the first fragments of slice s + 1.
  // (Past the last slice the refill re-reads the last columns and the writes and requests touch a buffer
  // that nobody uses: no branches in the step.)
  constexpr int kSteps = kTileK / 16, kLandSlots = (kSteps - 1) * FM, kPieces = Shape::kLandX + Shape::kLandY;
  static_assert(FM == FN, "two fragments per slot");
  static_assert(kPieces <= 2 * kLandSlots, "at most two register pieces per slot");
#define PLC_PIECE(p)                                                                            \
  if ((p) < Shape::kLandX) {                                                                    \
    *reinterpret_cast<uint4 *>(&xn[lp * SX + l_lane + row_of((p), wave) * 8]) = px[(p)];        \
    px[(p)] = fetch_x((p), koff);                                                               \
  } else if ((p) < kPieces) {                                                                   \
    *reinterpret_cast<uint4 *>(&yn[lp * SY + l_lane + row_of((p)-Shape::kLandX, wave) * 8]) =   \
        py[(p)-Shape::kLandX];                                                                  \
    py[(p)-Shape::kLandX] = fetch_y((p)-Shape::kLandX, koff);                                   \
  }
#pragma unroll
  for (int a = 0; a < FM; ++a) {
    fa[0][a] = *reinterpret_cast<const half8 *>(&gemm_lds[frag_x + a * 32 * 8]);
    fb[0][a] = *reinterpret_cast<const half8 *>(&gemm_lds[8 * SX + frag_y + a * 32 * 8]);
  }
  for (int s = 0; s < slices; ++s) {
    const int cur = s & 1;
    const _Float16 *const xs = gemm_lds + cur * Shape::kBufHalves, *const ys = xs + 8 * SX;
    _Float16 *const xn = gemm_lds + (cur ^ 1) * Shape::kBufHalves, *const yn = xn + 8 * SX;
    const unsigned koff = (unsigned)min(head + (s + 1) * kTileK + k_mine, k_last);  // slice s + 2
#pragma unroll
    for (int ks = 0; ks < kSteps; ++ks) {
      if (ks == kSteps - 1) __syncthreads();
#pragma unroll
      for (int a = 0; a < FM; ++a) {
        const int slot = ks * FM + a;
        if (ks + 1 < kSteps) {
          fa[(ks + 1) & 1][a] = *reinterpret_cast<const half8 *>(&xs[frag_x + 2 * (ks + 1) * SX + a * 32 * 8]);
          fb[(ks + 1) & 1][a] = *reinterpret_cast<const half8 *>(&ys[frag_y + 2 * (ks + 1) * SY + a * 32 * 8]);
          PLC_PIECE(slot);
          PLC_PIECE(slot + kLandSlots);
        } else {
          fa[0][a] = *reinterpret_cast<const half8 *>(&xn[frag_x + a * 32 * 8]);
          fb[0][a] = *reinterpret_cast<const half8 *>(&yn[frag_y + a * 32 * 8]);
        }
        __builtin_amdgcn_sched_barrier(0);  // memory instructions stay ahead of this slot's products
#pragma unroll
        for (int b = 0; b < FN; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[ks & 1][a], fb[ks & 1][b], acc[a][b], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
#undef PLC_PIECE

  const int row0 = tile_m * Shape::kTileM + wm * FM * 32 + 4 * (lane >> 5);
  const int col0 = tile_n * Shape::kTileN + wn * FN * 32 + (lane & 31);
#pragma unroll
  for (int a = 0; a < FM; ++a)
#pragma unroll
    for (int b = 0; b < FN; ++b)
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

// Launches over a (tiles, batches) grid.  The large tile is taken when the output divides into it and leaves
// at least one workgroup per compute unit; otherwise the small one.  The LDS buffers exceed 64 KB, which a
// kernel has to be granted before its launch.
template <class Shape, class Epilogue>
void launch_shape(int64_t M, int64_t N, int batches, hipStream_t st, const _Float16 *X, const _Float16 *Y, int64_t xs,
                  int64_t ys, int32_t xdiv, int32_t ymod, int K, const Epilogue &ep) {
  (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_nt_kernel<Shape, Epilogue>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)Shape::kLdsBytes);
  const int tiles_n = (int)(N / Shape::kTileN);
  const dim3 grid((unsigned)((M / Shape::kTileM) * tiles_n), (unsigned)batches);
  hipLaunchKernelGGL((gemm_nt_kernel<Shape, Epilogue>), grid, dim3(Shape::kThreads), Shape::kLdsBytes, st, X, Y, xs, ys,
                     xdiv, ymod, K, tiles_n, ep);
}

template <class Epilogue>
void launch_gemm(int64_t M, int64_t N, int batches, hipStream_t st, const _Float16 *X, const _Float16 *Y, int64_t xs,
                 int64_t ys, int32_t xdiv, int32_t ymod, int K, const Epilogue &ep) {
  const bool large = M % LargeTile::kTileM == 0 && N % LargeTile::kTileN == 0 &&
                     (M / LargeTile::kTileM) * (N / LargeTile::kTileN) * batches >= 256;
  if (large)
    launch_shape<LargeTile>(M, N, batches, st, X, Y, xs, ys, xdiv, ymod, K, ep);
  else
    launch_shape<SmallTile>(M, N, batches, st, X, Y, xs, ys, xdiv, ymod, K, ep);
}

bool aligned16(const void *p) { return p && (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool linear_shapes_ok(const plc_dims *dm, int32_t m) {
  if (!dm || dm->S < 1 || dm->L < 1 || dm->H < 1) return false;
  if (dm->n < SmallTile::kTileM || dm->n % SmallTile::kTileM) return false;                    // positions: whole tiles of rows
  if (dm->d < 8 || dm->d % 8 || (2 * dm->H * dm->d) % SmallTile::kTileN) return false;  // (head, K/V, component): whole tiles
  if (m < SmallTile::kTileN || m % SmallTile::kTileN) return false;
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
  if (rows < SmallTile::kTileM || rows % SmallTile::kTileM || m < SmallTile::kTileN || m % SmallTile::kTileN || V < 32 || V % 32) return PLC_ERR_INVALID;
  const int64_t tiles = (rows / SmallTile::kTileM) * (m / SmallTile::kTileN);
  if (tiles >= (1ll << 31)) return PLC_ERR_INVALID;
  StoreHalf ep{static_cast<_Float16 *>(ebar), m};
  hipStream_t st = static_cast<hipStream_t>(stream);
  {
    TraceScope trace(PLC_TRACE_EXPECTED_EMBEDDING, st);
    launch_gemm(rows, m, 1, st, static_cast<const _Float16 *>(probs_full), static_cast<const _Float16 *>(embed_t),
                (int64_t)0, (int64_t)0, 1, 1, V, ep);
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
    launch_gemm(dims->n, N, dims->S * dims->L, st, static_cast<const _Float16 *>(ebar),
                static_cast<const _Float16 *>(A), (int64_t)dims->n * m, (int64_t)N * m, dims->L, dims->L, m, ep);
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
    launch_gemm(dims->n, N, dims->S * dims->L, st, static_cast<const _Float16 *>(ebar),
                static_cast<const _Float16 *>(A), (int64_t)dims->n * m, (int64_t)N * m, dims->L, dims->L, m, ep);
  }
  if (hipGetLastError() != hipSuccess) return PLC_ERR_HIP;
  return patch_escapes(dims, symbols, esc_vals, esc_len, esc_off, out_k, out_v, ws, ws_bytes, status, st);
}
