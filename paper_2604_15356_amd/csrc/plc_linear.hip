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
// Both are C[M, N] = X[M, K] * Y[N, K]^T with fp16 operands, K contiguous in both, and fp32 accumulation
// in v_mfma_f32_32x32x16_f16.  A workgroup of WM x WN wavefronts owns a tile of C, each wavefront FM x FN
// MFMA tiles of 32 x 32 of it, and K advances in slices of 64 through LDS.  Two kernels share this plan:
//   - 256 x 256 tiles whose slices the memory system writes straight into LDS (used whenever the output
//     divides into such tiles and there is at least one per compute unit);
//   - 128 x 128 tiles whose slices pass through registers, for the small shapes.
// In both, the memory instructions of the slices to come are spread between the products of the current
// one, and the accumulators reach the epilogue through LDS, eight consecutive columns per lane.
#include "plc_device.h"

namespace plc {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int kTileK = 64;

// ---- slices through registers -------------------------------------------------------------------
//
// While slice s is multiplied, slice s + 1 moves from registers to the other of two LDS buffers and slice
// s + 2 from global memory into those registers, one piece at a time between the products; one barrier per
// slice.
//
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

// Hands a wavefront's accumulators to the epilogue eight consecutive columns at a time.  In the MFMA's
// result layout a lane owns one column of a 32 x 32 tile; the values of 32 rows of the wavefront's tile go
// through LDS (which the multiply no longer needs: the caller has passed a barrier) and come back with each
// lane owning eight consecutive columns of one row, so that the epilogue moves 16 bytes per operand and lane.
template <int FM, int FN, class Epilogue>
__device__ __forceinline__ void emit_tile(float16v (&acc)[FM][FN], float *lds, int wave, int lane, int batch, int row0,
                                          int col0, const Epilogue &ep) {
  constexpr int W = FN * 32, RS = W + 4;       // columns of the wavefront's tile; row stride in floats
  constexpr int kLanesPerRow = W / 8, kRowsPerPass = 64 / kLanesPerRow;
  float *const stage = lds + wave * (32 * RS);
  const int wr = 4 * (lane >> 5) * RS + (lane & 31);
  const int rd_row = lane / kLanesPerRow, rd_col = (lane % kLanesPerRow) * 8;
#pragma unroll
  for (int a = 0; a < FM; ++a) {
#pragma unroll
    for (int b = 0; b < FN; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) stage[wr + (8 * (i >> 2) + (i & 3)) * RS + b * 32] = acc[a][b][i];
#pragma unroll
    for (int pass = 0; pass < 32 / kRowsPerPass; ++pass) {
      const int r = pass * kRowsPerPass + rd_row;
      const float4 lo = *reinterpret_cast<const float4 *>(&stage[r * RS + rd_col]);
      const float4 hi = *reinterpret_cast<const float4 *>(&stage[r * RS + rd_col + 4]);
      const float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      ep(batch, row0 + a * 32 + r, col0 + rd_col, v);
    }
  }
}

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

  __syncthreads();  // every wavefront is done with the slices in LDS
  static_assert(Shape::kWaves * 32 * (FN * 32 + 4) * sizeof(float) <= Shape::kLdsBytes, "the output stage fits");
  emit_tile<FM, FN>(acc, reinterpret_cast<float *>(gemm_lds), wave, lane, batch, tile_m * Shape::kTileM + wm * FM * 32,
                    tile_n * Shape::kTileN + wn * FN * 32, ep);
}

// ---- the same contraction with direct global -> LDS loads ---------------------------------------
//
// K advances in slices of 64 through a ring of two or three LDS buffers that the memory system fills directly
// (16 bytes per lane; lane l of a load lands at the load's LDS base + 16 l), so a slice costs neither
// registers nor LDS write instructions.  One load moves a block of 8 rows x 128 bytes, eight consecutive
// lanes fetching one row (whole cache lines).  Inside a block the eight 16-byte pieces of row r are stored
// permuted, piece p in slot p ^ r (the lane of slot t fetches piece t ^ r), and the two blocks of a pair
// lie 128 bytes further apart than their size: the 16 lanes that read one piece of 16 consecutive rows for
// a multiply fragment then touch 16 different bank groups.
//
// The loop turns at its barrier, which stands before the last K step of a slice.  There every wavefront has
// read its last fragment of slice s and has waited for its own loads of slice s + 1, so after the barrier
// slice s + 1 is complete, and the buffer of slice s is free and starts to receive the slice that comes
// a whole ring later.
template <int WM_, int WN_, int FM_, int FN_, int NB_>
struct DirectShape {
  static constexpr int kWavesM = WM_, kWavesN = WN_, kFragsM = FM_, kFragsN = FN_;
  static constexpr int kWaves = WM_ * WN_, kThreads = 64 * kWaves;
  static constexpr int kTileM = 32 * FM_ * WM_, kTileN = 32 * FN_ * WN_;
  static constexpr int kSliceK = 64, kSteps = kSliceK / 16, kBuffers = NB_;
  static constexpr int kBlocksX = kTileM / 8, kBlocksY = kTileN / 8;  // blocks of 1 KB per slice
  static constexpr int kLoads = (kBlocksX + kBlocksY) / kWaves;       // per wavefront and slice
  static constexpr int kPairBytes = 2 * 1024 + 128;                   // two blocks and the padding
  static constexpr int kBytesX = kBlocksX / 2 * kPairBytes, kBufBytes = (kBlocksX + kBlocksY) / 2 * kPairBytes;
  static constexpr size_t kLdsBytes = (size_t)kBuffers * kBufBytes;
  // The loads of a slice are issued from the barrier on, spread over this many K steps: three with three
  // buffers, two with two (the slice is needed at the next barrier; timed against one step: 2-6 % faster at
  // every K from 4096 to 50,048; four steps are 5-9 % slower).
  static constexpr int kLoadSteps = NB_ == 3 ? 3 : 2;
  static constexpr int kLoadsPerSlot = (kLoads + kLoadSteps * FM_ - 1) / (kLoadSteps * FM_);
  static_assert(NB_ == 2 || NB_ == 3, "ring of two or three buffers");
  static_assert(kLoads * kWaves == kBlocksX + kBlocksY, "whole loads per wavefront");
  static_assert((NB_ - 1) * kLoads < 64, "the loads in flight fit the counter");
  static_assert(kLdsBytes <= 160 * 1024, "LDS of a compute unit");
};
using DirectTile = DirectShape<2, 2, 4, 4, 2>;  // 256 x 256, 256 threads, two buffers

typedef __attribute__((address_space(3))) char lds_char;

// Waits until at most N of this wavefront's loads (and none of its LDS requests) are outstanding, then
// joins the workgroup's barrier.  The wait is written as the instruction itself so that the compiler's own
// bookkeeping of outstanding requests sees it; nothing that touches memory moves across.
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
  static_assert(N >= 0 && N < 64, "vmcnt has six bits");
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (0 << 8) | ((N >> 4) << 14));  // vmcnt(N) lgkmcnt(0)
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

template <class Shape, class Epilogue>
__global__ __launch_bounds__(Shape::kThreads) void gemm_nt_direct_kernel(const _Float16 *__restrict__ X,
                                                                         const _Float16 *__restrict__ Y,
                                                                         int64_t x_batch_stride, int64_t y_batch_stride,
                                                                         int32_t x_batch_div, int32_t y_batch_mod, int K,
                                                                         int tiles_n, Epilogue ep) {
  constexpr int FM = Shape::kFragsM, FN = Shape::kFragsN, NB = Shape::kBuffers, KS = Shape::kSteps;
  extern __shared__ __attribute__((aligned(1024))) char gemm_ring[];
  lds_char *const ring = (lds_char *)gemm_ring;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / Shape::kWavesN, wn = wave - wm * Shape::kWavesN;
  const int batch = blockIdx.y;
  const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x - tile_m * tiles_n;
  const _Float16 *xb = X + (int64_t)(batch / x_batch_div) * x_batch_stride + (int64_t)tile_m * Shape::kTileM * K;
  const _Float16 *yb = Y + (int64_t)(batch % y_batch_mod) * y_batch_stride + (int64_t)tile_n * Shape::kTileN * K;

  // load j of a wavefront moves block q = wave + kWaves * j of the slice (X blocks first, then Y blocks);
  // block q of an operand starts at (q / 2) * kPairBytes + (q % 2) * (1024 + 128)
  const int k_lane = ((lane & 7) ^ (lane >> 3)) * 8;  // the column, within a slice, of this lane's piece
  const unsigned g_lane = (unsigned)(lane >> 3) * (unsigned)K + (unsigned)k_lane;  // halves
  // Lanes whose column is not below `width` stay out of the load and leave their 16 bytes of LDS alone.
  auto request = [&](int j, int k0, int width, int buf) {
    const int q = wave + Shape::kWaves * j;
    const _Float16 *src = (q < Shape::kBlocksX ? xb + (int64_t)(8 * q) * K : yb + (int64_t)(8 * (q - Shape::kBlocksX)) * K);
    const int at = buf * Shape::kBufBytes + (q >> 1) * Shape::kPairBytes + (q & 1) * 1152;
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass of the compiler does not know the device's load-to-LDS builtin
    if (k_lane < width) __builtin_amdgcn_global_load_lds(src + (k0 + g_lane), ring + at, 16, 0, 0);
#else
    (void)src, (void)k0, (void)width, (void)at, (void)ring, (void)g_lane;
#endif
  };

  float16v acc[FM][FN];
#pragma unroll
  for (int a = 0; a < FM; ++a)
#pragma unroll
    for (int b = 0; b < FN; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

  // fragments: lane l holds row l % 32 of a group of 32 rows (four blocks, two pairs), K piece 2 ks + l / 32
  int frag_lane[KS];
  {
    const int r32 = lane & 31, j = r32 >> 3, r = r32 & 7, g = lane >> 5;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      frag_lane[ks] = (j >> 1) * Shape::kPairBytes + (j & 1) * 1152 + r * 128 + (((2 * ks + g) ^ r) << 4);
  }
  const int frag_x = wm * FM * 2 * Shape::kPairBytes;
  const int frag_y = Shape::kBytesX + wn * FN * 2 * Shape::kPairBytes;
  half8 fa[2][FM], fb[2][FN];

  // Slices: when K is an odd multiple of 32 the first slice is the short one (32 columns; the other half of
  // its LDS buffer is cleared first), so that every later slice is whole.  Requests past the last slice
  // repeat it into ring buffers that are no longer read, which keeps the count of outstanding loads the
  // same in every step.
  const int head = (K & (Shape::kSliceK - 1)) ? Shape::kSliceK / 2 : Shape::kSliceK;
  const int slices = 1 + (K - head) / Shape::kSliceK;
  auto k_of = [&](int t) {
    const int c = min(t, slices - 1);
    return c == 0 ? 0 : head + (c - 1) * Shape::kSliceK;
  };
  auto width_of = [&](int t) { return min(t, slices - 1) == 0 ? head : Shape::kSliceK; };
  if (head != Shape::kSliceK) {
    for (int i = threadIdx.x * 16; i < Shape::kBufBytes; i += Shape::kThreads * 16)
      *reinterpret_cast<uint4 *>(gemm_ring + i) = make_uint4(0u, 0u, 0u, 0u);
    __syncthreads();
  }
#pragma unroll
  for (int t = 0; t < NB; ++t)
#pragma unroll
    for (int j = 0; j < Shape::kLoads; ++j) request(j, k_of(t), width_of(t), t);
  wait_loads_and_barrier<(NB - 1) * Shape::kLoads>();

  // A K step has FM slots of FN products.  The fragments of the next K step are requested around the first
  // slot's products -- half of them right after, half before the second slot's -- so that they are several
  // slots old when the next step starts, and the wait in front of a step's first products covers no request
  // younger than that.  A slot may also issue loads of the slice a whole ring ahead.  Fences keep the memory
  // instructions out of the runs of products.  (Handing the order to the instruction scheduler as a sequence
  // of groups instead -- requests behind the step's first two products, a load behind each of the next --
  // was timed too: it mixes the products of neighbouring steps and waits for requests it has just made.)
  constexpr int kHalf = (FM + FN + 1) / 2;
  static_assert(FM >= 2, "two slots carry the fragment requests");
#define PLC_REQUEST_FRAGS(set, base, ks, e0, e1)                                                                  \
  _Pragma("unroll") for (int e = (e0); e < (e1); ++e) {                                                           \
    if (e < FN)                                                                                                   \
      fb[set][e] = *reinterpret_cast<const half8 *>((base) + frag_y + frag_lane[ks] + e * 2 * Shape::kPairBytes);  \
    else                                                                                                          \
      fa[set][e - FN] =                                                                                           \
          *reinterpret_cast<const half8 *>((base) + frag_x + frag_lane[ks] + (e - FN) * 2 * Shape::kPairBytes);    \
  }
  // K step ks of a slice: products of fragment set ks % 2; requests the fragments of step ks_next of the
  // slice in buffer `from` and, as the order-th step after the barrier (order < 0: none), its share of the
  // loads of slice fill_slice
#define PLC_LOADS(order, a, fill_slice)                                                                 \
  if ((order) >= 0 && (order) < Shape::kLoadSteps) {                                                    \
    _Pragma("unroll") for (int i = 0; i < Shape::kLoadsPerSlot; ++i) {                                  \
      const int idx = ((order)*FM + (a)) * Shape::kLoadsPerSlot + i;                                    \
      if (idx < Shape::kLoads) request(idx, k_of(fill_slice), width_of(fill_slice), (fill_slice) % NB); \
    }                                                                                                   \
  }
#define PLC_KSTEP(ks, from, ks_next, order, fill_slice)                                                 \
  _Pragma("unroll") for (int a = 0; a < FM; ++a) {                                                      \
    if (a == 1) {                                                                                       \
      PLC_REQUEST_FRAGS(((ks) + 1) & 1, from, ks_next, kHalf, FM + FN);                                 \
    }                                                                                                   \
    if (a > 0) {                                                                                        \
      PLC_LOADS(order, a, fill_slice);                                                                  \
    }                                                                                                   \
    __builtin_amdgcn_sched_barrier(0);                                                                  \
    _Pragma("unroll") for (int b = 0; b < FN; ++b) acc[a][b] =                                          \
        __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[(ks)&1][a], fb[(ks)&1][b], acc[a][b], 0, 0, 0);       \
    __builtin_amdgcn_sched_barrier(0);                                                                  \
    if (a == 0) {                                                                                       \
      PLC_REQUEST_FRAGS(((ks) + 1) & 1, from, ks_next, 0, kHalf);                                       \
      PLC_LOADS(order, a, fill_slice);                                                                  \
    }                                                                                                   \
  }
  static_assert(KS == 4, "the steps are written out below");
  {
    const char *const cur = gemm_ring;
    PLC_REQUEST_FRAGS(0, cur, 0, 0, FM + FN);
    PLC_KSTEP(0, cur, 1, -1, 0);
    PLC_KSTEP(1, cur, 2, -1, 0);
    PLC_KSTEP(2, cur, 3, -1, 0);
  }
  wait_loads_and_barrier<(NB - 2) * Shape::kLoads>();  // slice 1 has landed
  for (int s = 0; s + 1 < slices; ++s) {
    const char *const nxt = gemm_ring + ((s + 1) % NB) * Shape::kBufBytes;
    PLC_KSTEP(3, nxt, 0, 0, s + NB);
    PLC_KSTEP(0, nxt, 1, 1, s + NB);
    PLC_KSTEP(1, nxt, 2, 2, s + NB);
    PLC_KSTEP(2, nxt, 3, 3, s + NB);
    wait_loads_and_barrier<(NB - 2) * Shape::kLoads>();  // slice s + 2 has landed
  }
  {
    const char *const nxt = gemm_ring + (slices % NB) * Shape::kBufBytes;  // read, never used
    PLC_KSTEP(3, nxt, 0, -1, 0);
  }
#undef PLC_KSTEP
#undef PLC_LOADS
#undef PLC_REQUEST_FRAGS
  // nothing may still be writing this workgroup's LDS when it ends
  __builtin_amdgcn_s_waitcnt((7 << 4) | (15 << 8));  // vmcnt(0)

  __syncthreads();  // ... and every wavefront is done with the slices in LDS
  static_assert(Shape::kWaves * 32 * (FN * 32 + 4) * sizeof(float) <= Shape::kLdsBytes, "the output stage fits");
  emit_tile<FM, FN>(acc, reinterpret_cast<float *>(gemm_ring), wave, lane, batch, tile_m * Shape::kTileM + wm * FM * 32,
                    tile_n * Shape::kTileN + wn * FN * 32, ep);
}

// ---- epilogues --------------------------------------------------------------------------------

// An epilogue receives eight consecutive columns (col a multiple of 8) of one row of C.

typedef uint8_t byte8 __attribute__((ext_vector_type(8)));

struct StoreHalf {  // Ebar[row, col] = fp16(acc)
  _Float16 *out;
  int64_t ld;
  __device__ void operator()(int, int row, int col, const float (&v)[8]) const {
    half8 h;
#pragma unroll
    for (int j = 0; j < 8; ++j) h[j] = (_Float16)v[j];
    *reinterpret_cast<half8 *>(out + (int64_t)row * ld + col) = h;
  }
};

struct LinearCoord {
  int32_t L, H, n, d;
  int64_t as[4];
  // batch = s * L + l; col = (h * 2 + c) * d + e; d is a multiple of 8, so eight columns share (h, c)
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
  __device__ void operator()(int batch, int row, int col, const float (&v)[8]) const {
    int c;
    int64_t ao, so;
    g.locate(batch, row, col, &c, &ao, &so);
    const half8 bias = *reinterpret_cast<const half8 *>((c ? bias_v : bias_k) + ao);
    const half8 act = *reinterpret_cast<const half8 *>((c ? act_v : act_k) + ao);
    byte8 sym;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float pred = v[j] + (float)bias[j];
      const float r = (float)act[j] - pred;
      const float u = r / delta;
      const float qf = __builtin_rintf(u);
      sym[j] = __builtin_fabsf(qf) <= qmax ? (uint8_t)((int)qf + (int)kZeroSymbol) : (uint8_t)PLC_ESCAPE;
    }
    *reinterpret_cast<byte8 *>(symbols + so) = sym;
  }
};

struct DecodeLinear {  // c + A Ebar plus the dequantised residual (escaped components are patched by a later pass)
  LinearCoord g;
  const _Float16 *bias_k, *bias_v;
  _Float16 *out_k, *out_v;
  const uint8_t *symbols;
  float delta;
  __device__ void operator()(int batch, int row, int col, const float (&v)[8]) const {
    int c;
    int64_t ao, so;
    g.locate(batch, row, col, &c, &ao, &so);
    const half8 bias = *reinterpret_cast<const half8 *>((c ? bias_v : bias_k) + ao);
    const byte8 sym = *reinterpret_cast<const byte8 *>(symbols + so);
    half8 out;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float pred = v[j] + (float)bias[j];
      const float qf = (float)((int)sym[j] - (int)kZeroSymbol);
      float x = __builtin_fmaf(qf, delta, pred);
      asm("" : "+v"(x));  // round to fp32, then to fp16
      out[j] = (_Float16)x;
    }
    *reinterpret_cast<half8 *>((c ? out_v : out_k) + ao) = out;
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

template <class Shape, class Epilogue>
void launch_direct(int64_t M, int64_t N, int batches, hipStream_t st, const _Float16 *X, const _Float16 *Y, int64_t xs,
                   int64_t ys, int32_t xdiv, int32_t ymod, int K, const Epilogue &ep) {
  const int tiles_n = (int)(N / Shape::kTileN);
  const dim3 grid((unsigned)((M / Shape::kTileM) * tiles_n), (unsigned)batches);
  (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_nt_direct_kernel<Shape, Epilogue>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)Shape::kLdsBytes);
  hipLaunchKernelGGL((gemm_nt_direct_kernel<Shape, Epilogue>), grid, dim3(Shape::kThreads), Shape::kLdsBytes, st, X, Y, xs,
                     ys, xdiv, ymod, K, tiles_n, ep);
}

template <class Epilogue>
void launch_gemm(int64_t M, int64_t N, int batches, hipStream_t st, const _Float16 *X, const _Float16 *Y, int64_t xs,
                 int64_t ys, int32_t xdiv, int32_t ymod, int K, const Epilogue &ep) {
  const bool large = M % DirectTile::kTileM == 0 && N % DirectTile::kTileN == 0 &&
                     (M / DirectTile::kTileM) * (N / DirectTile::kTileN) * batches >= 256;
  if (large)
    launch_direct<DirectTile>(M, N, batches, st, X, Y, xs, ys, xdiv, ymod, K, ep);
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
      !aligned16(act_v) || !aligned16(symbols))
    return PLC_ERR_INVALID;
  hipStream_t st = static_cast<hipStream_t>(stream);
  // the escape pass's own checks (lists, workspace, status) before the contraction is enqueued
  if (int rc = gather_escapes(dims, act_k, act_v, symbols, esc_vals, esc_cap, esc_cnt, esc_off, ws, ws_bytes, status,
                              st, false))
    return rc;
  const int N = 2 * dims->H * dims->d;
  EncodeLinear ep{coord_of(dims),
                  static_cast<const _Float16 *>(bias_k),
                  static_cast<const _Float16 *>(bias_v),
                  static_cast<const _Float16 *>(act_k),
                  static_cast<const _Float16 *>(act_v),
                  symbols,
                  dims->delta,
                  (float)dims->qmax};
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
      !aligned16(out_v) || !aligned16(symbols))
    return PLC_ERR_INVALID;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (int rc = patch_escapes(dims, symbols, esc_vals, esc_len, esc_off, out_k, out_v, ws, ws_bytes, status, st, false))
    return rc;
  const int N = 2 * dims->H * dims->d;
  DecodeLinear ep{coord_of(dims),
                  static_cast<const _Float16 *>(bias_k),
                  static_cast<const _Float16 *>(bias_v),
                  static_cast<_Float16 *>(out_k),
                  static_cast<_Float16 *>(out_v),
                  symbols,
                  dims->delta};
  {
    TraceScope trace(PLC_TRACE_RECONSTRUCT_LINEAR, st);
    launch_gemm(dims->n, N, dims->S * dims->L, st, static_cast<const _Float16 *>(ebar),
                static_cast<const _Float16 *>(A), (int64_t)dims->n * m, (int64_t)N * m, dims->L, dims->L, m, ep);
  }
  if (hipGetLastError() != hipSuccess) return PLC_ERR_HIP;
  return patch_escapes(dims, symbols, esc_vals, esc_len, esc_off, out_k, out_v, ws, ws_bytes, status, st);
}
