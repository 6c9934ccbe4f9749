// GEMMs of the projections (QKV, O, MLP up/down, prefix, LM head):
//   out[M, N] = A[M, K] * W[N, K]^T  (+ bias, GELU, or split-K partial sums)
// bf16 mode: MFMA (v_mfma_f32_16x16x32_bf16), fp32 accumulation.  Prefill (many
// rows): 256 x 256 or 128 x 128 tiles staged through LDS.  Decode (<= 256 rows):
// K-slice kernels that stream the weights once, from a copy in fragment order.
// fp32 mode: an LDS-tiled VALU kernel (small models only).
// Both operands are K-contiguous, so a lane's MFMA fragment (8 consecutive k of
// one row) is one 16-byte load.  Up to two independent problems share a launch.
#include <algorithm>

#include "common.h"
#include "kernels.h"
#include "../../include/bt.h"

namespace bt {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
// 16 bytes in flight between global memory and LDS.  A native vector, not HIP's uint4 struct:
// arrays of the struct that live across loop iterations end up in private memory.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

struct GemmDesc {
  const void* A;
  const void* W;
  const float* bias;
  void* out;
  int M, N, K, lda, ldo, epi, splits;
  const void* A_lo;      // bf16 remainder plane of A (null: none)
  size_t out_lo_off;     // EPI_GELU: != 0 writes the output as hi / remainder planes
  const void* W_frag;    // W in MFMA fragment order (K-slice kernel)
  float2* row_max;       // per (column tile, row) candidates for argmax, or null
  const int32_t* lse_targets;   // EPI_LSE: per row the column whose value goes to lse_target_out
  float* lse_target_out;
  QkvEpilogue qe;               // EPI_QKV
  int tiles_m, tiles_n, tile_begin;   // tiles of this problem occupy blocks [tile_begin, tile_begin + tiles_m*tiles_n*splits)
};
struct GemmGroup {
  GemmDesc p[2];
  int n;
  bool stream_w;         // host side only: selects the kernel variant that streams the weights
};

// The decode (K-slice) kernels take a compact form of the same description: one 64-byte cache line
// per problem.  Every workgroup of a launch fetches its kernel arguments from memory before it can
// issue anything else, and each further line of arguments measurably lengthens that first trip.
// Implied: lda == K, ldo == N, tiles_n from N and the kernel's tile width; a missing second problem
// has tile_begin == INT_MAX.
struct alignas(64) KsDesc {
  const void* A;
  const void* W_frag;
  void* out;
  const float* bias;
  float2* row_max;
  int lo_delta;          // elements from A to its bf16 remainder plane (0: none)
  int M, N, K;
  int epi_splits;        // epi | splits << 8
  int tile_begin;
};
static_assert(sizeof(KsDesc) == 64, "one cache line per problem");
struct KsGroup {
  KsDesc p[2];
};
// The fields the kernel bodies use, under the names of GemmDesc.
struct KsView {
  const void* A;
  const void* A_lo;
  const void* W_frag;
  void* out;
  const float* bias;
  float2* row_max;
  int M, N, K, lda, ldo, epi, splits, tiles_n, tile_begin;
  __device__ __forceinline__ KsView(const KsDesc& c, int tile_cols)
      : A(c.A), A_lo(reinterpret_cast<const uint16_t*>(c.A) + c.lo_delta), W_frag(c.W_frag), out(c.out), bias(c.bias),
        row_max(c.row_max), M(c.M), N(c.N), K(c.K), lda(c.K), ldo(c.N), epi(c.epi_splits & 0xff),
        splits(c.epi_splits >> 8), tiles_n((c.N + tile_cols - 1) / tile_cols), tile_begin(c.tile_begin) {}
};

__device__ __forceinline__ float gelu_erf(float u) { return 0.5f * u * (1.0f + erff(u * 0.70710678118654752f)); }

// GELU for outputs that are kept to 16 bits (bf16 hi + remainder planes): erf by the rational
// approximation 7.1.26 of Abramowitz & Stegun, absolute error below 1.5e-7, a dozen operations
// instead of the library routine's several dozen.  The tiled GEMM epilogue applies it to 128
// elements per thread and tile, where the library erff cost as much as the tile's whole k loop.
// 1 + erf is formed without cancellation on the negative side.
__device__ __forceinline__ float gelu_erf_fast(float u) {
  const float z = fabsf(u) * 0.70710678118654752f;
  const float t = __frcp_rn(1.0f + 0.3275911f * z);
  const float poly = ((((1.061405429f * t - 1.453152027f) * t + 1.421413741f) * t - 0.284496736f) * t + 0.254829592f) * t;
  const float pe = poly * __expf(-z * z);                  // = erfc(z)
  return 0.5f * u * (u >= 0.f ? 2.0f - pe : pe);
}
template <class T> __device__ __forceinline__ float gelu_for(float u) { return gelu_erf(u); }
template <> __device__ __forceinline__ float gelu_for<bf16_t>(float u) { return gelu_erf_fast(u); }

// What an epilogue needs from the descriptor, as plain values (kept in registers).
struct EpiArgs {
  void* out;
  const float* bias;
  int M, N, ldo, epi;
  size_t out_lo_off;
  const int32_t* lse_targets;
  float* lse_target_out;
  float2* row_max;
  QkvEpilogue qe;
};
__device__ __forceinline__ EpiArgs epi_args(const GemmDesc& d) {
  return EpiArgs{d.out, d.bias, d.M, d.N, d.ldo, d.epi, d.out_lo_off, d.lse_targets, d.lse_target_out, d.row_max, d.qe};
}

template <class T>
__device__ __forceinline__ void epilogue_store(const EpiArgs& d, int split, int row, int col, float acc) {
  if (row >= d.M || col >= d.N) return;
  if (d.epi == EPI_PARTIAL) {
    reinterpret_cast<float*>(d.out)[((size_t)split * d.M + row) * d.N + col] = acc;
  } else {
    if (d.bias) acc += d.bias[col];
    if (d.epi == EPI_F32) reinterpret_cast<float*>(d.out)[(size_t)row * d.ldo + col] = acc;
    else store_act<T>(reinterpret_cast<T*>(d.out), (size_t)row * d.ldo + col, d.out_lo_off, gelu_for<T>(acc));
  }
}

// Four consecutive columns of one row (col a multiple of 4): one 16-byte store for float outputs,
// 8 bytes per plane for bf16.  The tiled kernels multiply with the weight fragment as the MFMA's
// first operand, so that a lane's four accumulator values are four neighbouring columns of one
// output row rather than four rows of one column: a quarter of the store instructions, and the
// bias arrives as one float4.  Needs N and ldo to be multiples of 4 (else the callers store
// element by element).
template <class T, int EPI>
__device__ __forceinline__ void epilogue_store4(const EpiArgs& d, int split, int row, int col, f32x4_t v) {
  if (row >= d.M || col >= d.N) return;
  if constexpr (EPI == EPI_PARTIAL) {
    *reinterpret_cast<float4*>(reinterpret_cast<float*>(d.out) + ((size_t)split * d.M + row) * d.N + col) = make_float4(v[0], v[1], v[2], v[3]);
  } else {
    if (d.bias) {
      const float4 b = *reinterpret_cast<const float4*>(d.bias + col);
      v[0] += b.x; v[1] += b.y; v[2] += b.z; v[3] += b.w;
    }
    const size_t o = (size_t)row * d.ldo + col;
    if constexpr (EPI == EPI_F32) *reinterpret_cast<float4*>(reinterpret_cast<float*>(d.out) + o) = make_float4(v[0], v[1], v[2], v[3]);
    else store_act4<T>(reinterpret_cast<T*>(d.out), o, d.out_lo_off, gelu_for<T>(v[0]), gelu_for<T>(v[1]), gelu_for<T>(v[2]), gelu_for<T>(v[3]));
  }
}

// The accumulator tiles of one wave, TM x TN MFMA results whose lane layout is (row lane%16, columns
// 4*(lane/16) + 0..3) relative to (row_base + 16 i, col_base + 16 j).  The epilogue kind is resolved
// once, outside the unrolled loops, so that each copy of the loop body stays small (a large body
// keeps the compiler from unrolling, and the accumulators then land in scratch memory).
template <class T, int TM, int TN>
__device__ __forceinline__ void epilogue_tiles(const EpiArgs& ea, int split, int row_base, int col_base, int lane,
                                               const f32x4_t (&acc)[TM][TN]) {
  const int row_l = lane & 15, col_l = (lane >> 4) * 4;
  if (ea.epi == EPI_QKV) {
    // Block-decoder prefill: q | k | v columns.  Rotary pairs column d with d + half inside a head's first
    // `rot` dims: with half == 8 the partner is the same accumulator element of lane ^ 32, with half == 16
    // the same lane's element of the neighbouring 16-column tile.  Every branch below depends on the tile
    // only (wave-uniform), so the shuffles are executed by all lanes.
    const QkvEpilogue& q = ea.qe;
    const int D = ea.N / 3, DH = q.d_head, half = q.rot >> 1;
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int row = row_base + i * 16 + row_l;
      const int rr = min(row, ea.M - 1);
      const int b = rr / q.n_new, pos = q.pos0 + (rr - b * q.n_new);
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col0 = col_base + j * 16;                  // first column of the tile (wave-uniform)
        if (col0 >= ea.N) continue;
        const int region = col0 / D, c0 = col0 - region * D;
        const int h = c0 / DH, d0 = c0 - h * DH;             // the tile's 16 columns lie in one head (DH % 16 == 0)
        const int col = col0 + col_l, d = d0 + col_l;
        const float4 bia = ea.bias ? *reinterpret_cast<const float4*>(ea.bias + col) : zero4;
        float v[4] = {acc[i][j][0] + bia.x, acc[i][j][1] + bia.y, acc[i][j][2] + bia.z, acc[i][j][3] + bia.w};
        if (region < 2 && d0 < q.rot) {
          float pv[4];
          if (half == 8) {
#pragma unroll
            for (int r = 0; r < 4; ++r) pv[r] = __shfl_xor(v[r], 32, kWave);
          } else {                                           // half == 16: tile j ^ 1 of this lane
            const float4 pb = ea.bias ? *reinterpret_cast<const float4*>(ea.bias + (col ^ 16)) : zero4;
            const f32x4_t pa = acc[i][j ^ 1];
            pv[0] = pa[0] + pb.x; pv[1] = pa[1] + pb.y; pv[2] = pa[2] + pb.z; pv[3] = pa[3] + pb.w;
          }
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int dd = d + r;
            const bool lo = dd < half;
            const float2 cs = q.rope[(size_t)pos * half + (lo ? dd : dd - half)];
            v[r] = lo ? v[r] * cs.x - pv[r] * cs.y : v[r] * cs.x + pv[r] * cs.y;
          }
        }
        if (row < ea.M) {
          if (region == 0) {
            *reinterpret_cast<float4*>(reinterpret_cast<float*>(ea.out) + (size_t)row * ea.ldo + col) = make_float4(v[0], v[1], v[2], v[3]);
          } else {
            T* cache = reinterpret_cast<T*>(region == 1 ? q.Kc : q.Vc);
            store_act4<T>(cache, ((size_t)(b * q.n_heads + h) * q.n_cap + pos) * DH + d, 0, v[0], v[1], v[2], v[3]);
          }
        }
      }
    }
    return;
  }
  if (ea.epi == EPI_LSE) {
    // Log-sum-exp pieces instead of the values: this wave holds, for each of its 16 * TM rows, 16 * TN
    // consecutive columns (TN / 4 groups of 64); the four lanes that share a row combine by shuffles.
    static_assert(TN % 4 == 0, "a wave covers whole 64-column groups");
    float2* stats = reinterpret_cast<float2*>(ea.out);
    const int groups = (ea.N + 63) >> 6;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int row = row_base + i * 16 + row_l;
      const int tgt = (row < ea.M && ea.lse_targets) ? ea.lse_targets[row] : -1;
#pragma unroll
      for (int jg = 0; jg < TN / 4; ++jg) {
        const int group = (col_base >> 6) + jg;
        float v[4][4];
        float m = -INFINITY;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int col = col_base + (jg * 4 + j) * 16 + col_l + r;
            const float x = acc[i][jg * 4 + j][r] + ((ea.bias && col < ea.N) ? ea.bias[col] : 0.f);
            v[j][r] = col < ea.N ? x : -INFINITY;
            m = fmaxf(m, v[j][r]);
            if (col == tgt) ea.lse_target_out[row] = x;
          }
        m = fmaxf(m, __shfl_xor(m, 16, kWave));
        m = fmaxf(m, __shfl_xor(m, 32, kWave));
        float ssum = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int r = 0; r < 4; ++r) ssum += v[j][r] > -INFINITY ? __expf(v[j][r] - m) : 0.f;
        ssum += __shfl_xor(ssum, 16, kWave);
        ssum += __shfl_xor(ssum, 32, kWave);
        if (lane < 16 && row < ea.M && group < groups) stats[(size_t)row * groups + group] = make_float2(m, ssum);
      }
    }
    return;
  }
  if (((ea.N | ea.ldo) & 3) != 0) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          epilogue_store<T>(ea, split, row_base + i * 16 + row_l, col_base + j * 16 + col_l + r, acc[i][j][r]);
    return;
  }
  if (ea.epi == EPI_PARTIAL) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        epilogue_store4<T, EPI_PARTIAL>(ea, split, row_base + i * 16 + row_l, col_base + j * 16 + col_l, acc[i][j]);
  } else if (ea.epi == EPI_F32) {
    if (ea.out) {                    // null: the caller wants the argmax candidates only
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          epilogue_store4<T, EPI_F32>(ea, split, row_base + i * 16 + row_l, col_base + j * 16 + col_l, acc[i][j]);
    }
    if (ea.row_max) {
      // argmax candidates: per row the largest value of this wave's 64 columns and its column, the
      // lowest on ties: own 16 values first (ascending columns), then the four lanes that share the row
      static_assert(TN % 4 == 0, "a wave covers whole 64-column groups");
      const int groups = (ea.N + 63) >> 6;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = row_base + i * 16 + row_l;
#pragma unroll
        for (int jg = 0; jg < TN / 4; ++jg) {
          const int group = (col_base >> 6) + jg;
          float bv = -INFINITY;
          int bi = 0x7fffffff;
#pragma unroll
          for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int col = col_base + (jg * 4 + j) * 16 + col_l + r;
              const float x = acc[i][jg * 4 + j][r] + ((ea.bias && col < ea.N) ? ea.bias[col] : 0.f);
              const bool take = (col < ea.N) & (x > bv);
              bv = take ? x : bv;
              bi = take ? col : bi;
            }
#pragma unroll
          for (int o = 16; o <= 32; o <<= 1) {
            const float ov = __shfl_xor(bv, o, kWave);
            const int oi = __shfl_xor(bi, o, kWave);
            const bool take = (ov > bv) | ((ov == bv) & (oi < bi));
            bv = take ? ov : bv;
            bi = take ? oi : bi;
          }
          if (lane < 16 && row < ea.M && group < groups) ea.row_max[(size_t)row * groups + group] = make_float2(bv, __int_as_float(bi));
        }
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        epilogue_store4<T, EPI_GELU>(ea, split, row_base + i * 16 + row_l, col_base + j * 16 + col_l, acc[i][j]);
  }
}

// ---------------------------------------------------------------------------
// Epilogue of a wave that owns a 16 TM x 64 patch, with the stores turned through LDS.  In the MFMA result layout a store instruction covers 16 rows x 64 bytes
// (fp32) or 16 rows x 32 bytes (a bf16 plane): a quarter or a half of a cache line per row, and the
// output traffic of a tile with few k-steps then costs as much as its multiplies.  Here every row tile
// (16 x 64 floats, finished: bias, GELU or rotary applied) goes to the wave's own LDS strip and comes
// back with the lanes running along the rows, so that a store instruction writes whole rows of the
// patch: 256 bytes (fp32) or 128 bytes (a bf16 plane, 16 bytes per lane) per row.  Only the wave
// itself touches its strip and a wave's LDS operations complete in order, so no barrier is needed.
// Preconditions (checked by epilogue_through_lds, else the register epilogue is used): col_base a
// multiple of 64, N % 8 == 0, ldo % 8 == 0; EPI_QKV: D a multiple of 64.
// ---------------------------------------------------------------------------
// 16-byte store with the streaming hint: an output row is written once and read by a later launch, so it
// should not displace the operand tiles the other workgroups of the XCD are still reading from L2.
__device__ __forceinline__ void store16_stream(void* p, uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  __builtin_nontemporal_store(u32x4_t{a, b, c, d}, reinterpret_cast<u32x4_t*>(p));
}
constexpr int kEpiLd = 64 + 4;                  // floats per strip row: the pad keeps the 16-byte writes of 8 rows on distinct banks
__device__ __forceinline__ bool epilogue_through_lds(const EpiArgs& ea) {
  return ea.epi != EPI_LSE && (ea.N & 7) == 0 && (ea.ldo & 7) == 0 && (ea.out_lo_off & 7) == 0 &&
         (ea.epi != EPI_QKV || (ea.N / 3) % 64 == 0);
}
template <int TM, int KIND>
__device__ __forceinline__ void epilogue_patch_lds(const EpiArgs& ea, int split, int row_base, int col_base, int lane,
                                                   const f32x4_t (&acc)[TM][4], float* ws) {
  constexpr int LD = kEpiLd, NJ = 4;
  const int row_l = lane & 15, col_l = (lane >> 4) * 4;
  const QkvEpilogue& q = ea.qe;
  const int D = ea.N / 3, DH = q.d_head, half = q.rot >> 1;
  const int region = KIND == EPI_QKV ? col_base / D : 0;                 // q, k or v: the patch lies in one of them
  const int c_reg = col_base - region * D;                               // column inside the region
  float4 bias[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int col = col_base + j * 16 + col_l;
    bias[j] = (KIND != EPI_PARTIAL && ea.bias && col < ea.N) ? *reinterpret_cast<const float4*>(ea.bias + col) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    // ---- finished values of row tile i into the strip, in the MFMA layout (row lane % 16, 4 columns per tile)
    int pos = 0;
    if constexpr (KIND == EPI_QKV) {
      const int rr = min(row_base + i * 16 + row_l, ea.M - 1);
      pos = q.pos0 + rr % q.n_new;
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const f32x4_t a = acc[i][j];
      float v[4] = {a[0] + bias[j].x, a[1] + bias[j].y, a[2] + bias[j].z, a[3] + bias[j].w};
      if constexpr (KIND == EPI_GELU) {
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = gelu_erf_fast(v[r]);
      }
      if constexpr (KIND == EPI_QKV) {
        const int d0 = (c_reg + j * 16) % DH;                            // first dim of the tile inside its head (wave-uniform)
        if (region < 2 && d0 < q.rot) {
          float pv[4];
          if (half == 8) {
#pragma unroll
            for (int r = 0; r < 4; ++r) pv[r] = __shfl_xor(v[r], 32, kWave);
          } else {                                                       // half == 16: tile j ^ 1 of this lane
            const f32x4_t pa = acc[i][j ^ 1];
            const float4 pb = bias[j ^ 1];
            pv[0] = pa[0] + pb.x; pv[1] = pa[1] + pb.y; pv[2] = pa[2] + pb.z; pv[3] = pa[3] + pb.w;
          }
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int dd = d0 + col_l + r;
            const bool lo = dd < half;
            const float2 cs = q.rope[(size_t)pos * half + (lo ? dd : dd - half)];
            v[r] = lo ? v[r] * cs.x - pv[r] * cs.y : v[r] * cs.x + pv[r] * cs.y;
          }
        }
      }
      *reinterpret_cast<float4*>(ws + row_l * LD + j * 16 + col_l) = make_float4(v[0], v[1], v[2], v[3]);
    }
    // ---- back out with the lanes along the rows
    const bool as_f32 = KIND == EPI_F32 || KIND == EPI_PARTIAL || (KIND == EPI_QKV && region == 0);
    if (as_f32) {
      constexpr int LPR = 16, RPI = 64 / LPR;                            // lanes per row, rows per instruction
      const int c = (lane % LPR) * 4, col = col_base + c;
#pragma unroll
      for (int p = 0; p < 16 / RPI; ++p) {
        const int rr = RPI * p + lane / LPR, row = row_base + i * 16 + rr;
        const float4 v = *reinterpret_cast<const float4*>(ws + rr * LD + c);
        if (row < ea.M && col < ea.N) {
          float* o = reinterpret_cast<float*>(ea.out) + (KIND == EPI_PARTIAL ? ((size_t)split * ea.M + row) * ea.N + col : (size_t)row * ea.ldo + col);
          store16_stream(o, __float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w));
        }
      }
    } else {
      constexpr int LPR = 8, RPI = 64 / LPR;
      const int c = (lane % LPR) * 8, col = col_base + c;
#pragma unroll
      for (int p = 0; p < 16 / RPI; ++p) {
        const int rr = RPI * p + lane / LPR, row = row_base + i * 16 + rr;
        const float4 x = *reinterpret_cast<const float4*>(ws + rr * LD + c);
        const float4 y = *reinterpret_cast<const float4*>(ws + rr * LD + c + 4);
        const float f[8] = {x.x, x.y, x.z, x.w, y.x, y.y, y.z, y.w};
        uint32_t hb[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) hb[e] = float_to_bf16_bits(f[e]);
        const uint4 hi = make_uint4(hb[0] | (hb[1] << 16), hb[2] | (hb[3] << 16), hb[4] | (hb[5] << 16), hb[6] | (hb[7] << 16));
        if (row < ea.M && col < ea.N) {
          if constexpr (KIND == EPI_QKV) {                               // k or v: the block KV cache, [b][h][slot][DH]
            const int b = row / q.n_new, slot = q.pos0 + (row - b * q.n_new);
            const int h = (c_reg + c) / DH, dd = (c_reg + c) - h * DH;
            uint16_t* cache = reinterpret_cast<uint16_t*>(region == 1 ? q.Kc : q.Vc);
            store16_stream(cache + ((size_t)(b * q.n_heads + h) * q.n_cap + slot) * DH + dd, hi.x, hi.y, hi.z, hi.w);
          } else {
            uint16_t* o = reinterpret_cast<uint16_t*>(ea.out) + (size_t)row * ea.ldo + col;
            store16_stream(o, hi.x, hi.y, hi.z, hi.w);
            if (ea.out_lo_off) {
              uint32_t lb[8];
#pragma unroll
              for (int e = 0; e < 8; ++e) lb[e] = float_to_bf16_bits(f[e] - bf16_bits_to_float(hb[e]));
              store16_stream(o + ea.out_lo_off, lb[0] | (lb[1] << 16), lb[2] | (lb[3] << 16), lb[4] | (lb[5] << 16), lb[6] | (lb[7] << 16));
            }
          }
        }
      }
    }
  }
}

// All epilogue kinds of a patch: through LDS where the shapes allow, else from the registers.
template <int TM>
__device__ __forceinline__ void epilogue_patch(const EpiArgs& ea, int split, int row_base, int col_base, int lane,
                                               const f32x4_t (&acc)[TM][4], float* ws) {
  if (epilogue_through_lds(ea)) {
    if (ea.epi == EPI_GELU) epilogue_patch_lds<TM, EPI_GELU>(ea, split, row_base, col_base, lane, acc, ws);
    else if (ea.epi == EPI_PARTIAL) epilogue_patch_lds<TM, EPI_PARTIAL>(ea, split, row_base, col_base, lane, acc, ws);
    else if (ea.epi == EPI_QKV) epilogue_patch_lds<TM, EPI_QKV>(ea, split, row_base, col_base, lane, acc, ws);
    else {
      if (ea.out)                      // null: the caller wants the argmax candidates only
        epilogue_patch_lds<TM, EPI_F32>(ea, split, row_base, col_base, lane, acc, ws);
      if (ea.row_max) {                // the argmax candidates come from the registers
        EpiArgs ec = ea;
        ec.out = nullptr;
        epilogue_tiles<bf16_t, TM, 4>(ec, split, row_base, col_base, lane, acc);
      }
    }
    return;
  }
  epilogue_tiles<bf16_t, TM, 4>(ea, split, row_base, col_base, lane, acc);
}

// ---------------------------------------------------------------------------
// bf16 MFMA kernel.  256 threads = 4 waves laid out WM x WN over a BM x BN tile,
// BK = 64 per stage.  Global -> registers -> LDS with the next stage's loads in
// flight while the current stage is multiplied.
// ---------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN, bool HL>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmGroup g) {
  constexpr int BK = 64;
  constexpr int LDS = BK + 8;                   // row stride in elements (pad against bank conflicts)
  constexpr int TM = BM / WM / 16, TN = BN / WN / 16;
  constexpr int A_CH = BM * (BK / 8) / 256;     // 16-byte chunks per thread
  constexpr int B_CH = BN * (BK / 8) / 256;
  static_assert(WM * WN == 4 && A_CH >= 1 && B_CH >= 1, "tile shape");
  __shared__ __attribute__((aligned(16))) uint16_t sA[BM * LDS];
  __shared__ __attribute__((aligned(16))) uint16_t sAl[HL ? BM * LDS : 8];
  __shared__ __attribute__((aligned(16))) uint16_t sB[BN * LDS];

  const int bid = blockIdx.x;
  GemmDesc d = g.p[0];
  if (g.n > 1 && bid >= g.p[1].tile_begin) d = g.p[1];
  const EpiArgs ea = epi_args(d);
  int t = bid - d.tile_begin;
  const int T = d.tiles_m * d.tiles_n;
  const int split = t / T;
  t -= split * T;
  // Tile order.  Workgroups are dealt to the 8 XCDs round-robin and each XCD has its own L2, so
  // XCD x takes a contiguous run of the tile list (t -> start(x) + t / 8); the list itself walks
  // kGroupM row tiles down, then one column tile across.  The workgroups resident on an XCD at
  // one time thus cover a compact patch of the output and share their A and W tiles in its L2.
  {
    constexpr int kXcd = 8, kGroupM = 8;
    const int x = t % kXcd, q = T / kXcd, rem = T % kXcd;
    t = x * q + min(x, rem) + t / kXcd;
    const int per_group = kGroupM * d.tiles_n;
    const int grp = t / per_group, within = t - grp * per_group;
    const int gm = min(kGroupM, d.tiles_m - grp * kGroupM);
    t = (grp * kGroupM + within % gm) + (within / gm) * d.tiles_m;      // = tm + tn * tiles_m
  }
  const int tm_idx = t % d.tiles_m, tn_idx = t / d.tiles_m;
  const int m0 = tm_idx * BM, n0 = tn_idx * BN;
  const int Ks = d.K / d.splits;
  const int k_begin = split * Ks;
  const int KT = Ks / BK;

  const uint16_t* A = reinterpret_cast<const uint16_t*>(d.A);
  const uint16_t* W = reinterpret_cast<const uint16_t*>(d.W);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WM, wn = wave / WM;

  // per-thread global chunk coordinates
  const uint16_t* a_ptr[A_CH];
  const uint16_t* b_ptr[B_CH];
  int a_lds[A_CH], b_lds[B_CH];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int c = tid + i * 256, row = c >> 3, kc = c & 7;
    const int gr = min(m0 + row, d.M - 1);
    a_ptr[i] = A + (size_t)gr * d.lda + k_begin + kc * 8;
    a_lds[i] = row * LDS + kc * 8;
  }
  const ptrdiff_t lo_delta = HL ? reinterpret_cast<const uint16_t*>(d.A_lo) - A : 0;
#pragma unroll
  for (int i = 0; i < B_CH; ++i) {
    const int c = tid + i * 256, row = c >> 3, kc = c & 7;
    const int gr = min(n0 + row, d.N - 1);
    b_ptr[i] = W + (size_t)gr * d.K + k_begin + kc * 8;
    b_lds[i] = row * LDS + kc * 8;
  }

  f32x4_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  u32x4_t ra[A_CH], rb[B_CH], rl[HL ? A_CH : 1];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    ra[i] = *reinterpret_cast<const u32x4_t*>(a_ptr[i]);
    if constexpr (HL) rl[i] = *reinterpret_cast<const u32x4_t*>(a_ptr[i] + lo_delta);
  }
#pragma unroll
  for (int i = 0; i < B_CH; ++i) rb[i] = *reinterpret_cast<const u32x4_t*>(b_ptr[i]);

  const int frag_row = lane & 15, frag_k = (lane >> 4) * 8;
  for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      *reinterpret_cast<u32x4_t*>(&sA[a_lds[i]]) = ra[i];
      if constexpr (HL) *reinterpret_cast<u32x4_t*>(&sAl[a_lds[i]]) = rl[i];
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) *reinterpret_cast<u32x4_t*>(&sB[b_lds[i]]) = rb[i];
    __syncthreads();
    {
      // next stage (the last iteration re-reads its own stage: no branch around the loads)
      const size_t ko = (size_t)min(kt + 1, KT - 1) * BK;
#pragma unroll
      for (int i = 0; i < A_CH; ++i) {
        ra[i] = *reinterpret_cast<const u32x4_t*>(a_ptr[i] + ko);
        if constexpr (HL) rl[i] = *reinterpret_cast<const u32x4_t*>(a_ptr[i] + lo_delta + ko);
      }
#pragma unroll
      for (int i = 0; i < B_CH; ++i) rb[i] = *reinterpret_cast<const u32x4_t*>(b_ptr[i] + ko);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 32; ++ks) {
      bf16x8_t fa[TM], fb[TN], fl[HL ? TM : 1];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = wm * (BM / WM) + i * 16 + frag_row;
        fa[i] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(&sA[row * LDS + ks * 32 + frag_k]));
        if constexpr (HL) fl[i] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(&sAl[row * LDS + ks * 32 + frag_k]));
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int row = wn * (BN / WN) + j * 16 + frag_row;
        fb[j] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(&sB[row * LDS + ks * 32 + frag_k]));
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
          if constexpr (HL) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fl[i], acc[i][j], 0, 0, 0);
        }
    }
    __syncthreads();
  }

  // The weight fragment is the MFMA's first operand: the 16 x 16 result is the tile transposed, and a
  // lane holds output row lane%16, columns 4*(lane/16) + 0..3.  The loop's closing barrier has passed:
  // the four waves' strips (16 x 68 floats each) reuse the A tile.
  static_assert(TN == 4 && 4 * 16 * kEpiLd * 4 <= BM * LDS * 2, "one 64-column patch per wave; strips fit into sA");
  epilogue_patch<TM>(ea, split, m0 + wm * (BM / WM), n0 + wn * (BN / WN), lane, acc, reinterpret_cast<float*>(sA) + wave * (16 * kEpiLd));
}

// ---------------------------------------------------------------------------
// bf16 MFMA kernel for large M and N: 256 x 256 tile, BK = 64, 512 threads =
// 8 waves laid out 2 (rows) x 4 (columns), each wave a 128 x 64 patch
// (8 x 4 MFMA tiles).  A CU takes in operand bytes far more slowly than its
// matrix cores consume them, so the tile is as large as the register file
// allows: per byte loaded it does twice the work of the 128 x 128 tile.
// Global -> registers -> LDS, next stage in flight during the multiply.
// ---------------------------------------------------------------------------
template <bool HL>
__global__ __launch_bounds__(512) void gemm_bf16_big_kernel(GemmGroup g) {
  constexpr int BM = 256, BN = 256, BK = 64, LDS = BK + 8;
  constexpr int CH = BM * (BK / 8) / 512;       // 16-byte chunks per thread and operand plane (= 4)
  extern __shared__ __attribute__((aligned(16))) uint16_t sbig[];
  uint16_t* sA = sbig;
  uint16_t* sB = sbig + BM * LDS;
  uint16_t* sAl = sbig + (BM + BN) * LDS;       // only with HL

  const int bid = blockIdx.x;
  GemmDesc d = g.p[0];
  if (g.n > 1 && bid >= g.p[1].tile_begin) d = g.p[1];
  const EpiArgs ea = epi_args(d);
  int t = bid - d.tile_begin;
  const int T = d.tiles_m * d.tiles_n;
  const int split = t / T;
  t -= split * T;
  {   // same tile order as the 128 x 128 kernel: a contiguous run per XCD, 4 row tiles down then across
    constexpr int kXcd = 8, kGroupM = 4;
    const int x = t % kXcd, q = T / kXcd, rem = T % kXcd;
    t = x * q + min(x, rem) + t / kXcd;
    const int per_group = kGroupM * d.tiles_n;
    const int grp = t / per_group, within = t - grp * per_group;
    const int gm = min(kGroupM, d.tiles_m - grp * kGroupM);
    t = (grp * kGroupM + within % gm) + (within / gm) * d.tiles_m;
  }
  const int m0 = (t % d.tiles_m) * BM, n0 = (t / d.tiles_m) * BN;
  const int Ks = d.K / d.splits, k_begin = split * Ks, KT = Ks / BK;
  const uint16_t* A = reinterpret_cast<const uint16_t*>(d.A);
  const uint16_t* W = reinterpret_cast<const uint16_t*>(d.W);
  const ptrdiff_t lo_delta = HL ? reinterpret_cast<const uint16_t*>(d.A_lo) - A : 0;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1;

  // chunk c = tid + i * 512 -> row c >> 3, k-chunk c & 7 (rows 64 apart for consecutive i)
  const int ld_row = tid >> 3, ld_kc = tid & 7;
  const uint16_t* a_ptr[CH];
  const uint16_t* b_ptr[CH];
#pragma unroll
  for (int i = 0; i < CH; ++i) {
    a_ptr[i] = A + (size_t)min(m0 + ld_row + 64 * i, d.M - 1) * d.lda + k_begin + ld_kc * 8;
    b_ptr[i] = W + (size_t)min(n0 + ld_row + 64 * i, d.N - 1) * d.K + k_begin + ld_kc * 8;
  }
  const int lds_st = ld_row * LDS + ld_kc * 8;

  f32x4_t acc[8][4];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  u32x4_t ra[CH], rb[CH], rl[HL ? CH : 1];
#pragma unroll
  for (int i = 0; i < CH; ++i) {
    ra[i] = *reinterpret_cast<const u32x4_t*>(a_ptr[i]);
    if constexpr (HL) rl[i] = *reinterpret_cast<const u32x4_t*>(a_ptr[i] + lo_delta);
    rb[i] = *reinterpret_cast<const u32x4_t*>(b_ptr[i]);
  }
  const int frag_row = lane & 15, frag_k = (lane >> 4) * 8;
  const uint16_t* fa_base = sA + (wm * 128 + frag_row) * LDS + frag_k;
  const uint16_t* fb_base = sB + (wn * 64 + frag_row) * LDS + frag_k;
  for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      *reinterpret_cast<u32x4_t*>(&sA[lds_st + 64 * i * LDS]) = ra[i];
      if constexpr (HL) *reinterpret_cast<u32x4_t*>(&sAl[lds_st + 64 * i * LDS]) = rl[i];
      *reinterpret_cast<u32x4_t*>(&sB[lds_st + 64 * i * LDS]) = rb[i];
    }
    __syncthreads();
    {
      const size_t ko = (size_t)min(kt + 1, KT - 1) * BK;     // last iteration re-reads its own stage: no branch
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        ra[i] = *reinterpret_cast<const u32x4_t*>(a_ptr[i] + ko);
        if constexpr (HL) rl[i] = *reinterpret_cast<const u32x4_t*>(a_ptr[i] + lo_delta + ko);
        rb[i] = *reinterpret_cast<const u32x4_t*>(b_ptr[i] + ko);
      }
    }
#pragma unroll
    for (int ks = 0; ks < BK / 32; ++ks) {
      bf16x8_t fb[4];
#pragma unroll
      for (int j = 0; j < 4; ++j)
        fb[j] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(fb_base + j * 16 * LDS + ks * 32));
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const bf16x8_t fa = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(fa_base + i * 16 * LDS + ks * 32));
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa, acc[i][j], 0, 0, 0);
        if constexpr (HL) {
          const bf16x8_t fl = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(fa_base + (BM + BN) * LDS + i * 16 * LDS + ks * 32));
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fl, acc[i][j], 0, 0, 0);
        }
      }
    }
    __syncthreads();
  }
  // weight fragment first: a lane holds output row lane%16, columns 4*(lane/16) + 0..3 of each MFMA tile.
  // The loop's closing barrier has passed: the eight waves' strips (16 x 68 floats each) reuse the A tile.
  epilogue_patch<8>(ea, split, m0 + wm * 128, n0 + wn * 64, lane, acc, reinterpret_cast<float*>(sbig) + wave * (16 * kEpiLd));
}

// ---------------------------------------------------------------------------
// fp32 VALU kernel: 64 x 64 tile, BK = 16, each thread a 4 x 4 patch.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmGroup g) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float sA[BK][BM + 4];
  __shared__ float sB[BK][BN + 4];
  const int bid = blockIdx.x;
  GemmDesc d = g.p[0];
  if (g.n > 1 && bid >= g.p[1].tile_begin) d = g.p[1];
  const EpiArgs ea = epi_args(d);
  int t = bid - d.tile_begin;
  const int split = t / (d.tiles_m * d.tiles_n);
  t -= split * d.tiles_m * d.tiles_n;
  const int m0 = (t % d.tiles_m) * BM, n0 = (t / d.tiles_m) * BN;
  const int Ks = d.K / d.splits, k_begin = split * Ks;
  const float* A = reinterpret_cast<const float*>(d.A);
  const float* W = reinterpret_cast<const float*>(d.W);
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < Ks; k0 += BK) {
    for (int c = tid; c < BM * BK; c += 256) {
      const int row = c / BK, kk = c % BK;
      const int gr = m0 + row, gk = k0 + kk;
      sA[kk][row] = (gr < d.M && gk < Ks) ? A[(size_t)gr * d.lda + k_begin + gk] : 0.f;
    }
    for (int c = tid; c < BN * BK; c += 256) {
      const int row = c / BK, kk = c % BK;
      const int gr = n0 + row, gk = k0 + kk;
      sB[kk][row] = (gr < d.N && gk < Ks) ? W[(size_t)gr * d.K + k_begin + gk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = sA[kk][ty * 4 + i]; b[i] = sB[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) epilogue_store<float>(ea, split, m0 + ty * 4 + i, n0 + tx * 4 + j, acc[i][j]);
}

// ---------------------------------------------------------------------------
// bf16 kernel for skinny problems (M <= 256: decode steps).  These GEMMs are
// bound by reading W once from HBM, and a CU ingests only a few tens of GB/s,
// so the design goal is few bytes per workgroup and all of them in flight at
// once.  A workgroup owns 64*NT output columns (16*NT per wave) and a run of
// k_iters K-slices of 32*KF; per slice it stages the activation slice (all M
// rows, hi and lo planes) in LDS once for its four waves, while every wave holds
// its weight fragments in registers, loaded before anything else.  Each K-split
// writes raw partial sums [split][M][N]; the consumer adds bias / activation.
// With one split the usual epilogue (bias, GELU) is applied here.
// ---------------------------------------------------------------------------
// All-reduce over the 16 lanes of a DPP row by rotations (0x120 + n = rotate right by n inside
// the row): after steps 8, 4, 2, 1 every lane holds the result.  Register to register; a shuffle
// would go through the LDS crossbar.
template <int CTRL>
__device__ __forceinline__ float row_max_step(float v) {
  return fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false)));
}
template <int CTRL>
__device__ __forceinline__ int row_min_step(int v) {
  return min(v, __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false));
}

// One weight fragment (16 bytes per lane); STREAM: with the non-temporal hint (GemmProblem::stream_w).
template <bool STREAM>
__device__ __forceinline__ u32x4_t load_w_fragment(const uint16_t* p) {
  if constexpr (STREAM) return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  else return *reinterpret_cast<const u32x4_t*>(p);
}

template <int KF, int NT, int MC, bool HL, bool SW = false>
__global__ __launch_bounds__(256) void gemm_kslice_kernel(KsGroup g) {
  constexpr int KS = 32 * KF, LDK = KS + 8, CPR = KS / 8, PL = HL ? 2 : 1;
  extern __shared__ __attribute__((aligned(16))) uint16_t sA[];
  const int bid = blockIdx.x;
  // The descriptor is copied into registers at once: every field the epilogue needs is then
  // already there instead of being fetched from the argument block after the multiply.
  KsDesc c = g.p[0];
  if (bid >= g.p[1].tile_begin) c = g.p[1];
  const KsView d(c, 64 * NT);
  const int t = bid - d.tile_begin;
  const int split = t / d.tiles_n, tn = t - split * d.tiles_n;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n0 = tn * 64 * NT + wave * 16 * NT;
  const int Mpad = (d.M + 15) & ~15;
  const int k_iters = d.K / KS / d.splits;
  const int kblocks = d.K >> 5, last_tile = ((d.N + 15) >> 4) - 1;
  const uint16_t* A = reinterpret_cast<const uint16_t*>(d.A);
  const uint16_t* Wf = reinterpret_cast<const uint16_t*>(d.W_frag);
  const ptrdiff_t lo_delta = HL ? reinterpret_cast<const uint16_t*>(d.A_lo) - A : 0;

  f32x4_t acc[MC][NT][4];
#pragma unroll
  for (int mc = 0; mc < MC; ++mc)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) acc[mc][nt][mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const int total = Mpad * CPR;                 // 16-byte chunks of one plane of the slice
  for (int it = 0; it < k_iters; ++it) {
    const int kbase = (split * k_iters + it) * KS;
    // weight fragments of this wave: issued first, they come from HBM.  In fragment order the KF
    // fragments of one 16-column tile are KF consecutive KB.  Tiles past N repeat the last tile;
    // their products are never stored.
    bf16x8_t wf[NT][KF];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int tile = min((n0 >> 4) + nt, last_tile);
      const uint16_t* wp = Wf + ((size_t)tile * kblocks + (kbase >> 5)) * 512 + lane * 8;
#pragma unroll
      for (int kf = 0; kf < KF; ++kf) wf[nt][kf] = __builtin_bit_cast(bf16x8_t, load_w_fragment<SW>(wp + kf * 512));
    }
    // activation slice -> LDS.  No branches here: chunk indices past the end are clamped to the
    // last chunk (which is then loaded and stored more than once, with the same bytes), so the
    // compiler keeps all loads in flight together instead of sinking them into conditionals.
    // Rows past M repeat the last row; their products are never stored.
    for (int c0 = 0; c0 < total; c0 += 256 * 6) {
      uint4 r[PL][6];
      int lds_off[6];
#pragma unroll
      for (int u = 0; u < 6; ++u) {
        const int c = min(c0 + u * 256 + tid, total - 1);
        const int row = c / CPR, kc = c - row * CPR;
        const uint16_t* ap = A + (size_t)min(row, d.M - 1) * d.lda + kbase + kc * 8;
        lds_off[u] = row * LDK + kc * 8;
        r[0][u] = *reinterpret_cast<const uint4*>(ap);
        if constexpr (HL) r[1][u] = *reinterpret_cast<const uint4*>(ap + lo_delta);
      }
#pragma unroll
      for (int u = 0; u < 6; ++u) {
        *reinterpret_cast<uint4*>(&sA[lds_off[u]]) = r[0][u];
        if constexpr (HL) *reinterpret_cast<uint4*>(&sA[Mpad * LDK + lds_off[u]]) = r[1][u];
      }
    }
    __syncthreads();
    // Row tiles past the last one re-use its LDS rows (clamped, never stored), which keeps the
    // loops free of branches: the 4 * NT accumulator chains of a 64-row chunk interleave.
#pragma unroll
    for (int mc = 0; mc < MC; ++mc) {
#pragma unroll
      for (int kf = 0; kf < KF; ++kf) {
        bf16x8_t af[4], al[HL ? 4 : 1];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
          const int row = min(mc * 64 + mt * 16 + (lane & 15), Mpad - 1);
          const uint16_t* sp = &sA[row * LDK + (lane >> 4) * 8 + kf * 32];
          af[mt] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(sp));
          if constexpr (HL) al[mt] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(sp + Mpad * LDK));
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int mt = 0; mt < 4; ++mt)
            acc[mc][nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[mt], wf[nt][kf], acc[mc][nt][mt], 0, 0, 0);
        if constexpr (HL) {
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
              acc[mc][nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al[mt], wf[nt][kf], acc[mc][nt][mt], 0, 0, 0);
        }
      }
    }
    __syncthreads();
  }
  if (d.epi == EPI_PARTIAL) {
    float* outp = reinterpret_cast<float*>(d.out) + (size_t)split * d.M * d.N;
#pragma unroll
    for (int mc = 0; mc < MC; ++mc)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
          const int col = n0 + nt * 16 + (lane & 15);
          const int row0 = mc * 64 + mt * 16 + (lane >> 4) * 4;
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (row0 + r < d.M && col < d.N) outp[(size_t)(row0 + r) * d.N + col] = acc[mc][nt][mt][r];
        }
    return;
  }
  // Candidates first: the barrier inside would otherwise wait for the logit stores to drain.
  if (d.row_max) {
    // Per row: best (value, column) of this workgroup's 64*NT columns, lowest column on ties.
    // A lane holds rows 4 (lane >> 4) + r of each 16-row tile and one column per 16-column tile:
    // first over its own columns, then over the 16 lanes that share the rows, then over the waves.
    float bcol[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int col = n0 + nt * 16 + (lane & 15);
      bcol[nt] = (d.bias && col < d.N) ? d.bias[col] : 0.f;
    }
    float* red_v = reinterpret_cast<float*>(sA);            // [4 waves][64 MC rows]; the slice is no longer needed
    int* red_i = reinterpret_cast<int*>(sA) + 4 * 64 * MC;
#pragma unroll
    for (int mc = 0; mc < MC; ++mc)
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          // own columns first (ascending, so the lowest column wins ties), then the row's maximum
          // over the 16 lanes, then the lowest column among the lanes that hold it
          float bv = -INFINITY;
          int bi = 0x7fffffff;
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            const int col = n0 + nt * 16 + (lane & 15);
            const float v = acc[mc][nt][mt][r] + bcol[nt];
            const bool take = (col < d.N) & (v > bv);
            bv = take ? v : bv;
            bi = take ? col : bi;
          }
          float mx = bv;
          mx = row_max_step<0x128>(mx); mx = row_max_step<0x124>(mx); mx = row_max_step<0x122>(mx); mx = row_max_step<0x121>(mx);
          bi = (bv == mx) ? bi : 0x7fffffff;
          bi = row_min_step<0x128>(bi); bi = row_min_step<0x124>(bi); bi = row_min_step<0x122>(bi); bi = row_min_step<0x121>(bi);
          bv = mx;
          if ((lane & 15) == 0) {
            const int row = mc * 64 + mt * 16 + (lane >> 4) * 4 + r;
            red_v[wave * 64 * MC + row] = bv;
            red_i[wave * 64 * MC + row] = bi;
          }
        }
    __syncthreads();
    for (int row = tid; row < d.M; row += 256) {
      float bv = red_v[row];
      int bi = red_i[row];
#pragma unroll
      for (int w = 1; w < 4; ++w) {
        const float ov = red_v[w * 64 * MC + row];
        const int oi = red_i[w * 64 * MC + row];
        const bool take = (ov > bv) | ((ov == bv) & (oi < bi));
        bv = take ? ov : bv;
        bi = take ? oi : bi;
      }
      d.row_max[(size_t)row * d.tiles_n + tn] = make_float2(bv, __int_as_float(bi));
    }
  }
  // EPI_F32 (the launcher admits nothing else here): out = acc + bias, float; a null out means the
  // caller wants the candidates only
  if (d.out) {
    float* outp = reinterpret_cast<float*>(d.out);
#pragma unroll
    for (int mc = 0; mc < MC; ++mc)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
          const int col = n0 + nt * 16 + (lane & 15);
          const int row0 = mc * 64 + mt * 16 + (lane >> 4) * 4;
          const float bcol = (d.bias && col < d.N) ? d.bias[col] : 0.f;
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (row0 + r < d.M && col < d.N) outp[(size_t)(row0 + r) * d.ldo + col] = acc[mc][nt][mt][r] + bcol;
        }
  }
}

// The K-slice kernel as a software pipeline over two LDS buffers, for launches whose
// workgroups walk several 64-element K-slices (a single slice works too): while slice it
// is multiplied out of one buffer, the registers holding slice it + 1 are written to the
// other and refilled with slice it + 2 from global memory, one 256-thread chunk per
// multiply step, so the loads, the LDS stores and the matrix instructions of a wave
// interleave instead of taking turns (one workgroup per CU at 129-256 rows: nobody else
// would fill the gaps).  One barrier per slice.  The K-slices of a problem are dealt to
// its splits as evenly as they go.  hi + remainder planes only; EPI_PARTIAL or EPI_F32
// without argmax candidates; MC * KF <= 8 (registers: a whole slice is held by the 256
// threads); LDS: twice the slice, and a 16-row strip per wave for the epilogue.
// ---------------------------------------------------------------------------
constexpr int kPipeWaveRows = 1;               // waves along the rows of the workgroup's tile: 1 or 2 (measured equal)

template <int KF, int NT, int MC, bool SW = false, int WM = kPipeWaveRows>
__global__ __launch_bounds__(256) void gemm_kslice_pipe_kernel(KsGroup g) {
  constexpr int KS = 32 * KF, LDK = KS + 8, CPR = KS / 8, NCH = MC * KF;
  // the four waves as WM x (4 / WM) over the workgroup's rows and columns: a wave multiplies
  // MCW 64-row chunks by NTW 16-column tiles
  constexpr int MCW = MC / WM, NTW = NT * WM;
  static_assert(MC % WM == 0 && (WM == 1 || WM == 2), "wave grid");
  extern __shared__ __attribute__((aligned(16))) uint16_t sA[];
  const int bid = blockIdx.x;
  KsDesc c = g.p[0];
  if (bid >= g.p[1].tile_begin) c = g.p[1];
  const KsView d(c, 64 * NT);
  const int t = bid - d.tile_begin;
  const int split = t / d.tiles_n, tn = t - split * d.tiles_n;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave % WM, wave_n = wave / WM;
  const int n0 = tn * 64 * NT + wave_n * 16 * NTW;
  const int m0 = wave_m * 64 * MCW;
  const int Mpad = (d.M + 15) & ~15;
  // the K-slices of a problem are dealt to its splits as evenly as they go: the first
  // (slices % splits) splits walk one slice more
  const int slices = d.K / KS, q = slices / d.splits, rem = slices - q * d.splits;
  const int k_iters = q + (split < rem ? 1 : 0);
  const int kblocks = d.K >> 5, last_tile = ((d.N + 15) >> 4) - 1;
  const uint16_t* A = reinterpret_cast<const uint16_t*>(d.A);
  const uint16_t* Wf = reinterpret_cast<const uint16_t*>(d.W_frag);
  const ptrdiff_t lo_delta = reinterpret_cast<const uint16_t*>(d.A_lo) - A;

  f32x4_t acc[MCW][NTW][4];
#pragma unroll
  for (int mc = 0; mc < MCW; ++mc)
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) acc[mc][nt][mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // this thread's chunks of a slice: global offset (without the slice's k base) and LDS offset
  const int total = Mpad * CPR;
  int a_off[NCH], lds_off[NCH];
#pragma unroll
  for (int u = 0; u < NCH; ++u) {
    const int c = min(u * 256 + tid, total - 1);          // clamped: duplicates carry the same bytes
    const int row = c / CPR, kc = c - row * CPR;
    a_off[u] = min(row, d.M - 1) * d.lda + kc * 8;
    lds_off[u] = row * LDK + kc * 8;
  }
  const uint16_t* w_base[NTW];
#pragma unroll
  for (int nt = 0; nt < NTW; ++nt)
    w_base[nt] = Wf + (size_t)min((n0 >> 4) + nt, last_tile) * kblocks * 512 + lane * 8;

  // Order within a slice: MC * KF multiply steps; step s reads the fragments of step s + 1,
  // hands chunk s of slice it + 1 to LDS and reloads its registers with chunk s of slice
  // it + 2 (the last slice again once there is no further one: same bytes, harmless).
  constexpr int STEPS = MCW * KF, CPS = NCH / STEPS;      // CPS staged chunks per multiply step
  const int plane = Mpad * LDK;                    // elements of one plane; a buffer holds two
  const int slice0 = split * q + min(split, rem);
  u32x4_t wn[NTW][KF], ah[NCH], al[NCH];
  bf16x8_t wf[NTW][KF];
  {
    const int kbase = slice0 * KS;
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
      for (int kf = 0; kf < KF; ++kf)
        wf[nt][kf] = __builtin_bit_cast(bf16x8_t, load_w_fragment<SW>(w_base[nt] + (size_t)((kbase >> 5) + kf) * 512));
#pragma unroll
    for (int u = 0; u < NCH; ++u) {
      ah[u] = *reinterpret_cast<const u32x4_t*>(A + a_off[u] + kbase);
      al[u] = *reinterpret_cast<const u32x4_t*>(A + a_off[u] + kbase + lo_delta);
    }
#pragma unroll
    for (int u = 0; u < NCH; ++u) {
      *reinterpret_cast<u32x4_t*>(&sA[lds_off[u]]) = ah[u];
      *reinterpret_cast<u32x4_t*>(&sA[plane + lds_off[u]]) = al[u];
    }
    const int kbase1 = (slice0 + min(1, k_iters - 1)) * KS;
#pragma unroll
    for (int u = 0; u < NCH; ++u) {
      ah[u] = *reinterpret_cast<const u32x4_t*>(A + a_off[u] + kbase1);
      al[u] = *reinterpret_cast<const u32x4_t*>(A + a_off[u] + kbase1 + lo_delta);
    }
  }
  __syncthreads();
  auto lds_frags = [&](const uint16_t* buf, int step, bf16x8_t (&f)[8]) {
    const int mc = step / KF, kf = step - mc * KF;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
      const int row = min(m0 + mc * 64 + mt * 16 + (lane & 15), Mpad - 1);
      const uint16_t* sp = buf + row * LDK + (lane >> 4) * 8 + kf * 32;
      f[mt] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(sp));
      f[4 + mt] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(sp + plane));
    }
  };
  for (int it = 0; it < k_iters; ++it) {
    const uint16_t* cur = sA + (it & 1) * 2 * plane;
    uint16_t* nxt = sA + ((it + 1) & 1) * 2 * plane;
    const int kb1 = (slice0 + min(it + 1, k_iters - 1)) * KS;
    const int kb2 = (slice0 + min(it + 2, k_iters - 1)) * KS;
    bf16x8_t fr[2][8];
    lds_frags(cur, 0, fr[0]);
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
      for (int kf = 0; kf < KF; ++kf) wn[nt][kf] = load_w_fragment<SW>(w_base[nt] + (size_t)((kb1 >> 5) + kf) * 512);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int step = 0; step < STEPS; ++step) {
      const int mc = step / KF, kf = step - mc * KF;
      if (step + 1 < STEPS) lds_frags(cur, step + 1, fr[(step + 1) & 1]);
#pragma unroll
      for (int u = step * CPS; u < (step + 1) * CPS; ++u) {
        *reinterpret_cast<u32x4_t*>(&nxt[lds_off[u]]) = ah[u];
        *reinterpret_cast<u32x4_t*>(&nxt[plane + lds_off[u]]) = al[u];
        ah[u] = *reinterpret_cast<const u32x4_t*>(A + a_off[u] + kb2);
        al[u] = *reinterpret_cast<const u32x4_t*>(A + a_off[u] + kb2 + lo_delta);
      }
#pragma unroll
      for (int pl = 0; pl < 2; ++pl)
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
          for (int mt = 0; mt < 4; ++mt)
            acc[mc][nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fr[step & 1][pl * 4 + mt], wf[nt][kf], acc[mc][nt][mt], 0, 0, 0);
      // issue order of the step: one memory instruction in the shadow of each matrix instruction
      // (a wave issues in order; a block of loads ahead of the multiplies would leave the matrix
      // unit idle while they queue)
      constexpr int MF = 8 * NTW;                  // matrix instructions of the step
      constexpr int MEM = 8 + 4 * CPS;             // fragment reads, LDS stores and global loads
      constexpr int PER = MF / MEM > 0 ? MF / MEM : 1;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, PER, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
#pragma unroll
      for (int i = 0; i < 2 * CPS; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, PER, 0);
        __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
      }
#pragma unroll
      for (int i = 0; i < 2 * CPS; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, PER, 0);
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, MF - PER * MEM, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
      for (int kf = 0; kf < KF; ++kf) wf[nt][kf] = __builtin_bit_cast(bf16x8_t, wn[nt][kf]);
    __syncthreads();
  }
  if (d.epi == EPI_PARTIAL) {
    float* outp = reinterpret_cast<float*>(d.out) + (size_t)split * d.M * d.N;
    if ((d.N & 3) == 0 && (reinterpret_cast<uintptr_t>(outp) & 15) == 0) {
      // whole rows: each 16-row piece of the wave's tile goes through a strip of LDS of the wave's
      // own (behind the two slice buffers), so that a store instruction writes 16 bytes per lane
      // and whole 64-byte (NTW = 1: the tile is 16 columns wide) or 128-byte row segments
      constexpr int LDP = 16 * NTW + 4;            // floats per strip row
      constexpr int LPR = 4 * NTW;                 // lanes per row (16 bytes each)
      constexpr int RPI = 64 / LPR;                // rows per store instruction
      float* strip = reinterpret_cast<float*>(sA + 4 * plane) + wave * (16 * LDP);
      const int srow = lane / LPR, scol = (lane % LPR) * 4;
#pragma unroll
      for (int mc = 0; mc < MCW; ++mc)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
          for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) strip[((lane >> 4) * 4 + r) * LDP + nt * 16 + (lane & 15)] = acc[mc][nt][mt][r];
#pragma unroll
          for (int h = 0; h < 16 / RPI; ++h) {
            const int row = m0 + mc * 64 + mt * 16 + h * RPI + srow;
            const f32x4_t v = *reinterpret_cast<const f32x4_t*>(&strip[(h * RPI + srow) * LDP + scol]);
            if (row < d.M && n0 + scol < d.N) *reinterpret_cast<f32x4_t*>(&outp[(size_t)row * d.N + n0 + scol]) = v;
          }
        }
      return;
    }
#pragma unroll
    for (int mc = 0; mc < MCW; ++mc)
#pragma unroll
      for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
          const int col = n0 + nt * 16 + (lane & 15);
          const int row0 = m0 + mc * 64 + mt * 16 + (lane >> 4) * 4;
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (row0 + r < d.M && col < d.N) outp[(size_t)(row0 + r) * d.N + col] = acc[mc][nt][mt][r];
        }
    return;
  }
  // EPI_F32 (the launcher admits nothing else here): out = acc + bias, float
  {
    float* outp = reinterpret_cast<float*>(d.out);
#pragma unroll
    for (int mc = 0; mc < MCW; ++mc)
#pragma unroll
      for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
          const int col = n0 + nt * 16 + (lane & 15);
          const int row0 = m0 + mc * 64 + mt * 16 + (lane >> 4) * 4;
          const float bcol = (d.bias && col < d.N) ? d.bias[col] : 0.f;
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (row0 + r < d.M && col < d.N) outp[(size_t)(row0 + r) * d.ldo + col] = acc[mc][nt][mt][r] + bcol;
        }
  }
}

// W[N, K] -> fragment order, one thread per 16-byte chunk.
__global__ __launch_bounds__(256) void pack_weights_kernel(const uint16_t* __restrict__ W, uint16_t* __restrict__ Wf, int N, int K, size_t n_chunks) {
  const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (c >= n_chunks) return;
  const int lane = (int)(c & 63);
  const size_t tile_kb = c >> 6;
  const int kblocks = K >> 5;
  const int kb = (int)(tile_kb % kblocks), tile = (int)(tile_kb / kblocks);
  const int n = tile * 16 + (lane & 15), k = kb * 32 + (lane >> 4) * 8;
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (n < N) v = *reinterpret_cast<const uint4*>(W + (size_t)n * K + k);
  *reinterpret_cast<uint4*>(Wf + c * 8) = v;
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
namespace {
enum { KIND_F32 = 0, KIND_TILE128 = 1, KIND_KSLICE = 2, KIND_TILE256 = 3 };
constexpr int kMaxSkinnyRows = 256;
constexpr int kNumCU = 256;

int f32_splits(int N, int K) {
  const int tiles = (N + 63) / 64;
  int best = 1;
  for (int s = 1; s <= 16; ++s) {
    if (K % s) continue;
    const int ks = K / s;
    if (ks % 16 || ks < 32) continue;
    best = s;
    if (tiles * s >= 512) break;
  }
  return best;
}

size_t kslice_lds_bytes(int M, int kf, bool hl) {
  const int Mpad = (M + 15) & ~15;
  return (size_t)Mpad * (32 * kf + 8) * 2 * (hl ? 2 : 1);
}
}  // namespace

bool gemm_qkv_epilogue_ok(int d_model, int d_head, int rot) {
  const int half = rot / 2;
  return d_model % 64 == 0 && d_head % 16 == 0 && (rot == 0 || ((half == 8 || half == 16) && rot <= d_head));
}

bool gemm_has_lse_epilogue(const GemmPlan& plan) { return plan.kind == KIND_TILE256 || plan.kind == KIND_TILE128; }

int gemm_row_max_tiles(const GemmProblem& p, const GemmPlan& plan) {
  // candidates come from the plain K-slice kernel only: every row of a workgroup in one 64*MC chunk
  // set, one K-split, final values in the epilogue
  if (p.epi != EPI_F32 || plan.splits[0] != 1) return 0;
  // the tiled MFMA kernels: one candidate per row and 64 columns (N a multiple of 4: their vector epilogue)
  if (plan.kind == KIND_TILE256 || plan.kind == KIND_TILE128) return (p.N & 3) || (p.ldo & 3) ? 0 : (p.N + 63) / 64;
  if (plan.kind != KIND_KSLICE || plan.mc >= 4) return 0;
  return (p.N + 64 * plan.nt - 1) / (64 * plan.nt);
}

size_t gemm_packed_elems(int N, int K) { return (size_t)((N + 15) & ~15) * K; }

hipError_t gemm_pack_weights(const void* W, void* W_frag, int N, int K, hipStream_t s) {
  if (!W || !W_frag || N <= 0 || K <= 0 || K % 32) return hipErrorInvalidValue;
  const size_t n_chunks = gemm_packed_elems(N, K) / 8;
  pack_weights_kernel<<<(unsigned)((n_chunks + 255) / 256), 256, 0, s>>>(
      reinterpret_cast<const uint16_t*>(W), reinterpret_cast<uint16_t*>(W_frag), N, K, n_chunks);
  return hipGetLastError();
}

hipError_t gemm_plan(int dtype, const GemmProblem* probs, int n_probs, GemmPlan* plan) {
  if (n_probs < 1 || n_probs > 2 || !plan) return hipErrorInvalidValue;
  int max_m = 0;
  for (int i = 0; i < n_probs; ++i) {
    const GemmProblem& p = probs[i];
    if (p.M <= 0 || p.N <= 0 || p.K <= 0) return hipErrorInvalidValue;
    if (dtype == BT_BF16 && (p.K % 64 || p.lda % 8)) return hipErrorInvalidValue;
    if (p.M != probs[0].M) return hipErrorInvalidValue;
    max_m = p.M > max_m ? p.M : max_m;
    plan->splits[i] = 1;
  }
  plan->kf = 0;
  plan->nt = 1;
  plan->mc = 1;
  plan->uneven = 0;
  const bool hl = probs[0].A_lo != nullptr;
  if (dtype == BT_F32) {
    plan->kind = KIND_F32;
    if (max_m <= kMaxSkinnyRows)
      for (int i = 0; i < n_probs; ++i)
        if (probs[i].epi == EPI_PARTIAL) plan->splits[i] = f32_splits(probs[i].N, probs[i].K);
    return hipSuccess;
  }
  if (max_m > kMaxSkinnyRows) {
    // 256 x 256 tiles when they still fill the GPU; otherwise 128 x 128
    long tiles256 = 0;
    for (int i = 0; i < n_probs; ++i) tiles256 += (long)((probs[i].M + 255) / 256) * ((probs[i].N + 255) / 256);
    plan->kind = tiles256 >= kNumCU ? KIND_TILE256 : KIND_TILE128;
    return hipSuccess;
  }

  // A wide problem that finishes its own epilogue (the LM head) at more than 192 rows: the K-slice
  // kernel would pull the whole activation matrix through L2 once per 128 columns (4 x the weight
  // bytes at 256 rows); 256 x 256 tiles halve that (137 us against 204 us at 256 x 50304 x 2048).
  if (n_probs == 1 && probs[0].epi != EPI_PARTIAL && max_m > 192 && probs[0].N >= 4096) {
    plan->kind = KIND_TILE256;
    return hipSuccess;
  }
  // K-slice kernel.  Slice length: the longest of 256/192/128/64 that divides every K and keeps
  // the staged activation slice within the LDS budget below.
  plan->kind = KIND_KSLICE;
  plan->mc = (max_m + 63) / 64;
  if (plan->mc == 3) plan->mc = 4;
  // Plain kernel: up to 128 rows the slice stays within 64 KB (two workgroups per CU overlap their
  // phases).  With more rows one workgroup per CU walks many slices and overlaps load and multiply
  // itself (pipelined kernel), which needs mc * kf <= 8; the two-plane partial-sum launches with
  // fewer rows are moved to that kernel, with 64-element slices, further down.
  const size_t lds_cap = max_m <= 128 ? 64 * 1024 : 144 * 1024;
  int kf = 2;
  for (int c : {8, 6, 4, 2}) {
    bool ok = kslice_lds_bytes(max_m, c, hl) <= lds_cap && (max_m <= 128 || !hl || plan->mc * c <= 8);
    for (int i = 0; i < n_probs && ok; ++i) ok = probs[i].K % (32 * c) == 0;
    if (ok) { kf = c; break; }
  }
  plan->kf = kf;
  // Columns per workgroup (64*nt) and K-slices per workgroup (q): minimise the bytes a launch
  // moves (weights once, activation slices once per workgroup, partial sums written and read
  // back), stretched when there are too few workgroups to overlap each other's load, multiply
  // and store phases (measured: below about 1.75 workgroups per CU a launch is latency-bound).
  // Problems that must finish their own epilogue keep all slices in one workgroup.
  double best_cost = 1e300;
  for (int nt : {4, 2, 1}) {
    if (nt * plan->mc > 8) continue;                       // accumulator registers
    for (int q : {1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64, 128}) {
      int spl[2] = {1, 1};
      int wgs = 0;
      double cost = 0;
      for (int i = 0; i < n_probs; ++i) {
        const GemmProblem& p = probs[i];
        const int tiles = (p.N + 64 * nt - 1) / (64 * nt), slices = p.K / (32 * kf);
        if (p.epi == EPI_PARTIAL) {
          int qi = q < slices ? q : slices;
          while (slices % qi) --qi;                        // largest divisor of slices <= q
          spl[i] = slices / qi;
        }
        wgs += tiles * spl[i];
        cost += (double)p.N * p.K * 2;                                     // weights
        cost += (double)tiles * p.M * p.K * (hl ? 4 : 2);                  // activation reads
        if (p.epi == EPI_PARTIAL) cost += (double)spl[i] * p.M * p.N * 8;  // partials out and back
      }
      // workgroups wanted: 1.75 per CU, so that they overlap each other's phases.  Where LDS or
      // registers leave room for one workgroup per CU, the launch runs in rounds of one per CU and
      // what counts is how full the last round is.
      if (kslice_lds_bytes(max_m, kf, hl) > 80 * 1024 || plan->mc >= 4) {
        const int rounds = (wgs + kNumCU - 1) / kNumCU;
        cost *= (double)rounds * kNumCU / wgs;
      } else if (wgs < kNumCU * 1.75) {
        cost *= kNumCU * 1.75 / wgs;
      }
      if (cost < best_cost) {
        best_cost = cost;
        plan->nt = nt;
        plan->splits[0] = spl[0];
        plan->splits[1] = spl[1];
      }
    }
  }
  // The pipelined kernel (two planes, 64-element slices) runs one workgroup per CU and deals
  // K-slices to splits unevenly, so the slices per workgroup need not divide the slice counts:
  // take the q (longest walk) that minimises  q * (time of a slice) + partial sums out and back,
  // with all workgroups in one round.  Measured on 256 x 2048 x {2048, 8192} in one launch:
  // 16 slices per workgroup on 160 CUs against 11 on 240.  At 129-256 rows it serves every launch
  // (the plan above stands unless a q is clearly shorter); with fewer rows only launches made of
  // partial-sum problems (the others leave argmax candidates, which the plain kernel writes), with
  // the slice length set to 64 here (cfg1, 64 rows: 430 -> 409 us per decode step against the plain
  // kernel's one-shot 192-element slices; longer walks with fewer partial planes 418; batch 1 and 4
  // on the same model: 341 -> 350 and 345 -> 358 us, hence not below 8 rows).
  bool all_partial = true;
  for (int i = 0; i < n_probs; ++i) all_partial &= probs[i].epi == EPI_PARTIAL;
  const bool rows256 = hl && plan->mc == 4 && kf == 2 && plan->nt <= 2;
  bool rows128 = hl && plan->mc == 2 && all_partial;
  bool rows64 = hl && plan->mc == 1 && max_m >= 8 && all_partial;     // below 8 rows the plain kernel's one slice per workgroup is faster
  for (int i = 0; i < n_probs; ++i) {
    rows128 &= probs[i].K % 64 == 0;
    rows64 &= probs[i].K % 64 == 0;
  }
  if (rows256 || rows128 || rows64) {
    const double slice_us[3] = {0, rows256 ? 1.3 : rows128 ? 0.7 : 0.35, rows256 ? 1.9 : rows128 ? 1.0 : 0.5};   // per 64-element slice at nt = 1, 2
    constexpr double kPartialBytesPerUs = 5e6;
    auto model = [&](int nt, const int* spl) {
      int q_max = 0;
      double bytes = 0;
      for (int i = 0; i < n_probs; ++i) {
        const int slices = probs[i].K / 64;
        q_max = std::max(q_max, (slices + spl[i] - 1) / spl[i]);
        if (probs[i].epi == EPI_PARTIAL) bytes += (double)spl[i] * probs[i].M * probs[i].N * 8;
      }
      return q_max * slice_us[nt] + bytes / kPartialBytesPerUs;
    };
    double best = rows256 ? model(plan->nt, plan->splits) : 1e300;
    int max_slices = 0;
    for (int i = 0; i < n_probs; ++i) max_slices = std::max(max_slices, probs[i].K / 64);
    const int nt_first = rows256 ? plan->nt : 2, nt_last = rows256 ? plan->nt : 1;
    for (int nt = nt_first; nt >= nt_last; --nt)
      for (int q = 1; q <= max_slices; ++q) {
        int spl[2] = {1, 1};
        int wgs = 0;
        for (int i = 0; i < n_probs; ++i) {
          const int slices = probs[i].K / 64, tiles = (probs[i].N + 64 * nt - 1) / (64 * nt);
          if (probs[i].epi == EPI_PARTIAL) spl[i] = (slices + q - 1) / q;
          wgs += tiles * spl[i];
        }
        if (wgs > kNumCU) continue;
        const double t = model(nt, spl);
        if (t < best * 0.97) {                             // keep the plan in hand unless this one is clearly shorter
          best = t;
          plan->nt = nt;
          plan->splits[0] = spl[0];
          plan->splits[1] = spl[1];
          plan->uneven = 1;
          plan->kf = 2;
        }
      }
  }
  return hipSuccess;
}

template <int BM, int BN>
static int fill_tiles(GemmGroup& g) {
  int begin = 0;
  for (int i = 0; i < g.n; ++i) {
    g.p[i].tiles_m = (g.p[i].M + BM - 1) / BM;
    g.p[i].tiles_n = (g.p[i].N + BN - 1) / BN;
    g.p[i].tile_begin = begin;
    begin += g.p[i].tiles_m * g.p[i].tiles_n * g.p[i].splits;
  }
  return begin;
}

// Compact form of the group for the K-slice kernels (tile width 64 * NT columns); returns the grid size.
static int pack_kslice(const GemmGroup& g, int tile_cols, KsGroup& k) {
  int begin = 0;
  for (int i = 0; i < 2; ++i) {
    KsDesc& c = k.p[i];
    if (i >= g.n) { c = KsDesc{}; c.tile_begin = 0x7fffffff; continue; }
    const GemmDesc& d = g.p[i];
    c.A = d.A; c.W_frag = d.W_frag; c.out = d.out; c.bias = d.bias; c.row_max = d.row_max;
    c.lo_delta = d.A_lo ? (int)(reinterpret_cast<const uint16_t*>(d.A_lo) - reinterpret_cast<const uint16_t*>(d.A)) : 0;
    c.M = d.M; c.N = d.N; c.K = d.K;
    c.epi_splits = d.epi | (d.splits << 8);
    c.tile_begin = begin;
    begin += (d.N + tile_cols - 1) / tile_cols * d.splits;
  }
  return begin;
}

// Kernels that take more dynamic LDS than the default limit get the limit raised once per model
// (gemm_prepare_kernels, called by bt_create with the model's device current): the attribute belongs
// to the device's copy of the function, and the launchers keep no state of their own.
static hipError_t raise_lds_limit(const void* fn) {
  return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
}

template <int KF, int NT, int MC, bool HL>
static hipError_t launch_kslice(GemmGroup& g, size_t lds, hipStream_t s) {
  KsGroup k;
  const int grid = pack_kslice(g, 64 * NT, k);
  if constexpr (HL) {                     // the streaming variants exist for the two-plane kernels only
    if (g.stream_w) {
      gemm_kslice_kernel<KF, NT, MC, HL, true><<<grid, 256, lds, s>>>(k);
      return hipSuccess;
    }
  }
  gemm_kslice_kernel<KF, NT, MC, HL><<<grid, 256, lds, s>>>(k);
  return hipSuccess;
}

template <int KF, int NT, int MC>
static hipError_t launch_kslice_pipe(GemmGroup& g, size_t lds, hipStream_t s) {
  KsGroup k;
  const int grid = pack_kslice(g, 64 * NT, k);
  // two LDS buffers (at 256 rows and 64-element slices: 2 x 72 KB of the CU's 160 KB)
  // ... and a strip of 16 rows per wave for the epilogue's whole-row stores
  const size_t bytes = 2 * lds + 4 * 16 * (16 * NT * kPipeWaveRows + 4) * sizeof(float);
  if (bytes > 160 * 1024) return hipErrorInvalidValue;
  if (g.stream_w) gemm_kslice_pipe_kernel<KF, NT, MC, true><<<grid, 256, bytes, s>>>(k);
  else gemm_kslice_pipe_kernel<KF, NT, MC><<<grid, 256, bytes, s>>>(k);
  return hipSuccess;
}

// The pipelined variant exists for these (kf, nt, mc); returns false when there is none.
static bool launch_kslice_pipe_any(GemmGroup& g, int kf, int nt, int mc, size_t lds, hipStream_t s, hipError_t* e) {
  switch (kf * 100 + nt * 10 + mc) {
    case 211: *e = launch_kslice_pipe<2, 1, 1>(g, lds, s); return true;
    case 221: *e = launch_kslice_pipe<2, 2, 1>(g, lds, s); return true;
    case 212: *e = launch_kslice_pipe<2, 1, 2>(g, lds, s); return true;
    case 222: *e = launch_kslice_pipe<2, 2, 2>(g, lds, s); return true;
    case 214: *e = launch_kslice_pipe<2, 1, 4>(g, lds, s); return true;
    case 224: *e = launch_kslice_pipe<2, 2, 4>(g, lds, s); return true;
    default: return false;
  }
}

template <int KF, bool HL>
static hipError_t launch_kslice_kf(GemmGroup& g, int nt, int mc, size_t lds, hipStream_t s) {
  const int key = nt * 10 + mc;
  switch (key) {
    case 11: return launch_kslice<KF, 1, 1, HL>(g, lds, s);
    case 12: return launch_kslice<KF, 1, 2, HL>(g, lds, s);
    case 14: return launch_kslice<KF, 1, 4, HL>(g, lds, s);
    case 21: return launch_kslice<KF, 2, 1, HL>(g, lds, s);
    case 22: return launch_kslice<KF, 2, 2, HL>(g, lds, s);
    case 24: return launch_kslice<KF, 2, 4, HL>(g, lds, s);
    case 41: return launch_kslice<KF, 4, 1, HL>(g, lds, s);
    case 42: return launch_kslice<KF, 4, 2, HL>(g, lds, s);
    default: return hipErrorInvalidValue;
  }
}

template <int KF, bool HL>
static hipError_t prepare_kslice_kf() {
  hipError_t e = hipSuccess;
  auto up = [&](const void* fn) { if (e == hipSuccess) e = raise_lds_limit(fn); };
  up(reinterpret_cast<const void*>(gemm_kslice_kernel<KF, 1, 1, HL>));
  up(reinterpret_cast<const void*>(gemm_kslice_kernel<KF, 1, 2, HL>));
  up(reinterpret_cast<const void*>(gemm_kslice_kernel<KF, 1, 4, HL>));
  up(reinterpret_cast<const void*>(gemm_kslice_kernel<KF, 2, 1, HL>));
  up(reinterpret_cast<const void*>(gemm_kslice_kernel<KF, 2, 2, HL>));
  up(reinterpret_cast<const void*>(gemm_kslice_kernel<KF, 2, 4, HL>));
  up(reinterpret_cast<const void*>(gemm_kslice_kernel<KF, 4, 1, HL>));
  up(reinterpret_cast<const void*>(gemm_kslice_kernel<KF, 4, 2, HL>));
  if constexpr (HL) {
    up(reinterpret_cast<const void*>(gemm_kslice_kernel<KF, 1, 1, HL, true>));
    up(reinterpret_cast<const void*>(gemm_kslice_kernel<KF, 1, 2, HL, true>));
    up(reinterpret_cast<const void*>(gemm_kslice_kernel<KF, 1, 4, HL, true>));
    up(reinterpret_cast<const void*>(gemm_kslice_kernel<KF, 2, 1, HL, true>));
    up(reinterpret_cast<const void*>(gemm_kslice_kernel<KF, 2, 2, HL, true>));
    up(reinterpret_cast<const void*>(gemm_kslice_kernel<KF, 2, 4, HL, true>));
    up(reinterpret_cast<const void*>(gemm_kslice_kernel<KF, 4, 1, HL, true>));
    up(reinterpret_cast<const void*>(gemm_kslice_kernel<KF, 4, 2, HL, true>));
  }
  return e;
}

hipError_t gemm_prepare_kernels() {
  hipError_t e = hipSuccess;
  auto step = [&](hipError_t r) { if (e == hipSuccess) e = r; };
  step(prepare_kslice_kf<2, false>()); step(prepare_kslice_kf<2, true>());
  step(prepare_kslice_kf<4, false>()); step(prepare_kslice_kf<4, true>());
  step(prepare_kslice_kf<6, false>()); step(prepare_kslice_kf<6, true>());
  step(prepare_kslice_kf<8, false>()); step(prepare_kslice_kf<8, true>());
  step(raise_lds_limit(reinterpret_cast<const void*>(gemm_kslice_pipe_kernel<2, 1, 2>)));
  step(raise_lds_limit(reinterpret_cast<const void*>(gemm_kslice_pipe_kernel<2, 2, 2>)));
  step(raise_lds_limit(reinterpret_cast<const void*>(gemm_kslice_pipe_kernel<2, 1, 2, true>)));
  step(raise_lds_limit(reinterpret_cast<const void*>(gemm_kslice_pipe_kernel<2, 2, 2, true>)));
  step(raise_lds_limit(reinterpret_cast<const void*>(gemm_kslice_pipe_kernel<2, 1, 4>)));
  step(raise_lds_limit(reinterpret_cast<const void*>(gemm_kslice_pipe_kernel<2, 2, 4>)));
  step(raise_lds_limit(reinterpret_cast<const void*>(gemm_kslice_pipe_kernel<2, 1, 4, true>)));
  step(raise_lds_limit(reinterpret_cast<const void*>(gemm_kslice_pipe_kernel<2, 2, 4, true>)));
  step(raise_lds_limit(reinterpret_cast<const void*>(gemm_bf16_big_kernel<true>)));
  step(raise_lds_limit(reinterpret_cast<const void*>(gemm_bf16_big_kernel<false>)));
  return e;
}

hipError_t launch_gemm(int dtype, const GemmProblem* probs, int n_probs, const GemmPlan& plan, hipStream_t s) {
  if (n_probs < 1 || n_probs > 2) return hipErrorInvalidValue;
  GemmGroup g;
  g.n = n_probs;
  g.stream_w = probs[0].stream_w != 0;
  for (int i = 0; i < n_probs; ++i) {
    const GemmProblem& p = probs[i];
    const int sp = plan.splits[i];
    if (sp < 1 || (!plan.uneven && p.K % sp) || (sp > 1 && p.epi != EPI_PARTIAL)) return hipErrorInvalidValue;
    g.p[i].A = p.A; g.p[i].W = p.W; g.p[i].bias = p.bias; g.p[i].out = p.out;
    g.p[i].M = p.M; g.p[i].N = p.N; g.p[i].K = p.K; g.p[i].lda = p.lda; g.p[i].ldo = p.ldo;
    g.p[i].epi = p.epi; g.p[i].splits = sp;
    g.p[i].A_lo = p.A_lo; g.p[i].out_lo_off = p.out_lo_off; g.p[i].W_frag = p.W_frag; g.p[i].row_max = p.row_max;
    g.p[i].lse_targets = p.lse_targets; g.p[i].lse_target_out = p.lse_target_out;
    g.p[i].qe = p.qe;
    if (p.epi == EPI_QKV && ((plan.kind != KIND_TILE256 && plan.kind != KIND_TILE128) || sp != 1 || p.N % 3 ||
                             !gemm_qkv_epilogue_ok(p.N / 3, p.qe.d_head, p.qe.rot) || !p.qe.Kc || !p.qe.Vc || p.qe.n_new < 1))
      return hipErrorInvalidValue;
    if (p.epi == EPI_LSE && ((plan.kind != KIND_TILE256 && plan.kind != KIND_TILE128) || sp != 1 || !p.lse_target_out)) return hipErrorInvalidValue;
    if ((p.A_lo != nullptr) != (probs[0].A_lo != nullptr)) return hipErrorInvalidValue;
    if ((p.stream_w != 0) != (probs[0].stream_w != 0)) return hipErrorInvalidValue;
  }
  const bool hl = probs[0].A_lo != nullptr;
  if (hl && dtype != BT_BF16) return hipErrorInvalidValue;
  // Tiled kernels run in rounds of one (or two) tiles per CU, in block order.  With two problems whose
  // tiles cost differently (O: K = D, MLP-down: K = 4 D) the costly tiles go first, so that the last
  // round is made of cheap ones (348 tiles at 14 848 rows: 5 tile-times with O first, 4 with MLP-down first).
  if (n_probs == 2 && (plan.kind == KIND_TILE128 || plan.kind == KIND_TILE256) &&
      (long)g.p[1].K / g.p[1].splits > (long)g.p[0].K / g.p[0].splits) {
    const GemmDesc t = g.p[0];
    g.p[0] = g.p[1];
    g.p[1] = t;
  }
  switch (plan.kind) {
    case KIND_F32:
      gemm_f32_kernel<<<fill_tiles<64, 64>(g), 256, 0, s>>>(g);
      break;
    case KIND_TILE128:
      if (hl) gemm_bf16_kernel<128, 128, 2, 2, true><<<fill_tiles<128, 128>(g), 256, 0, s>>>(g);
      else gemm_bf16_kernel<128, 128, 2, 2, false><<<fill_tiles<128, 128>(g), 256, 0, s>>>(g);
      break;
    case KIND_TILE256: {
      const size_t lds = (size_t)(512 + (hl ? 256 : 0)) * 72 * 2;
      if (hl) gemm_bf16_big_kernel<true><<<fill_tiles<256, 256>(g), 512, lds, s>>>(g);
      else gemm_bf16_big_kernel<false><<<fill_tiles<256, 256>(g), 512, lds, s>>>(g);
      break;
    }
    case KIND_KSLICE: {
      for (int i = 0; i < n_probs; ++i) {
        const GemmProblem& p = probs[i];
        if (plan.uneven ? (p.K % (32 * plan.kf) || plan.splits[i] > p.K / (32 * plan.kf)) : p.K % (32 * plan.kf * plan.splits[i]))
          return hipErrorInvalidValue;
        if (!p.W_frag || p.epi == EPI_GELU) return hipErrorInvalidValue;
        // the compact argument form implies dense rows and a remainder plane within 2^31 elements
        if (p.lda != p.K || (p.epi == EPI_F32 && p.ldo != p.N) || plan.splits[i] > 0xffff) return hipErrorInvalidValue;
        if (p.A_lo) {
          const ptrdiff_t delta = reinterpret_cast<const uint16_t*>(p.A_lo) - reinterpret_cast<const uint16_t*>(p.A);
          if (delta <= 0 || delta > 0x7fffffff) return hipErrorInvalidValue;
        }
      }
      const size_t lds = kslice_lds_bytes(probs[0].M, plan.kf, hl);
      if (lds > 160 * 1024) return hipErrorInvalidValue;
      hipError_t e;
      bool several_slices = false;
      for (int i = 0; i < n_probs; ++i) several_slices |= probs[i].K / (32 * plan.kf * plan.splits[i]) >= 2;
      // The pipelined kernel serves every two-plane launch at 129-256 rows and, with fewer rows, the
      // launches the planner marked for it (partial-sum problems only: it leaves no argmax
      // candidates; the LM head at 64 rows was no faster on it than on the plain kernel, where
      // several workgroups per CU overlap each other's phases).
      bool all_partial = true;
      for (int i = 0; i < n_probs; ++i) all_partial &= probs[i].epi == EPI_PARTIAL;
      if (plan.mc <= 2 && plan.uneven && !all_partial) return hipErrorInvalidValue;
      if (hl && (several_slices || plan.uneven) && (plan.mc >= 4 || (plan.mc <= 2 && plan.uneven)) && launch_kslice_pipe_any(g, plan.kf, plan.nt, plan.mc, lds, s, &e)) {
        if (e != hipSuccess) return e;
        break;
      }
      if (plan.uneven) return hipErrorInvalidValue;   // only the pipelined kernel deals slices unevenly
      switch (plan.kf * 2 + (hl ? 1 : 0)) {
        case 4:  e = launch_kslice_kf<2, false>(g, plan.nt, plan.mc, lds, s); break;
        case 5:  e = launch_kslice_kf<2, true>(g, plan.nt, plan.mc, lds, s); break;
        case 8:  e = launch_kslice_kf<4, false>(g, plan.nt, plan.mc, lds, s); break;
        case 9:  e = launch_kslice_kf<4, true>(g, plan.nt, plan.mc, lds, s); break;
        case 12: e = launch_kslice_kf<6, false>(g, plan.nt, plan.mc, lds, s); break;
        case 13: e = launch_kslice_kf<6, true>(g, plan.nt, plan.mc, lds, s); break;
        case 16: e = launch_kslice_kf<8, false>(g, plan.nt, plan.mc, lds, s); break;
        case 17: e = launch_kslice_kf<8, true>(g, plan.nt, plan.mc, lds, s); break;
        default: e = hipErrorInvalidValue;
      }
      if (e != hipSuccess) return e;
      break;
    }
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace bt
