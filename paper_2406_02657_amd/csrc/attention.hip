// Attention kernels.
//   * block decoder, decode step (Sec. 2.3): one query per (sequence, head)
//     against the whole block-level KV cache - the memory-bound heart of the
//     step.  The cache rows of one (b, h) are contiguous, so a wavefront streams
//     them with 16-byte loads; the waves of a workgroup split the rows
//     (split-K) and merge their partial softmaxes through LDS.
//   * block decoder, prefill: causal attention over the prompt's blocks.
//   * token decoder (Sec. 2.4): attention inside the current block only; the
//     whole local KV of a (b, h) sits in LDS, reductions are wave shuffles.
// Scores, softmax and accumulation are fp32; K and V are read in storage dtype.
#include "common.h"
#include "kernels.h"
#include "../../include/bt.h"

namespace bt {

constexpr float kNegBig = -1.0e30f;

__device__ __forceinline__ float partial_value(const PartialSrc& p, size_t idx, int col) {
  float v = p.bias ? p.bias[col] : 0.f;
#pragma unroll 4
  for (int s = 0; s < p.splits; ++s) v += p.base[(size_t)s * p.stride + idx];
  return v;
}

__device__ __forceinline__ float gelu_erf_f(float u) { return 0.5f * u * (1.0f + erff(u * 0.70710678118654752f)); }

// Extra workgroups of an attention launch (or a launch of its own): block `blk` of `nblk`
// turns its share of the up-projection partial sums into the MLP hidden activation.
template <class T>
__device__ __forceinline__ void gelu_reduce_block(const GeluJob& j, int blk, int nblk) {
  const size_t groups = (size_t)j.rows * j.cols / 4;
  T* out = reinterpret_cast<T*>(j.out);
  for (size_t gi = (size_t)blk * blockDim.x + threadIdx.x; gi < groups; gi += (size_t)nblk * blockDim.x) {
    const size_t idx = gi * 4;
    const int col = (int)(idx % j.cols);
    float4 v = j.src.bias ? *reinterpret_cast<const float4*>(j.src.bias + col) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
    for (int s = 0; s < j.src.splits; ++s) {
      const float4 p = *reinterpret_cast<const float4*>(j.src.base + (size_t)s * j.src.stride + idx);
      v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
    }
    store_act4<T>(out, idx, j.out_lo_off, gelu_erf_f(v.x), gelu_erf_f(v.y), gelu_erf_f(v.z), gelu_erf_f(v.w));
  }
}

template <class T>
__global__ __launch_bounds__(256) void gelu_reduce_kernel(GeluJob j) { gelu_reduce_block<T>(j, blockIdx.x, gridDim.x); }

__host__ inline int gelu_blocks(const GeluJob& j) {
  if (j.rows <= 0) return 0;
  const size_t groups = (size_t)j.rows * j.cols / 4;
  size_t b = (groups + 255) / 256;            // one group of four activations per thread
  return (int)(b < 1 ? 1 : (b > 1024 ? 1024 : b));
}

template <class T, int DH>
struct RowMap {
  static constexpr int EPC = Chunk<T>::EPC;   // elements per 16-byte chunk
  static constexpr int LPR = DH / EPC;        // lanes per cache row
  static constexpr int RPL = kWave / LPR;     // rows per wave-wide load
};

// One wavefront attends one query to rows [j0, j1) of K, V ([row][DH]).
// Lane = (slot rr = lane / LPR, chunk sub = lane % LPR); q holds the lane's EPC
// query elements already scaled by 1/sqrt(DH).  Each slot runs an online
// softmax over its rows; at the end the slots are merged, so every lane
// returns the wave-wide (m, l, acc) for its chunk of dims.
// The row stream is double-buffered in registers: attend_issue() puts the loads
// of one batch (U row groups of K and of V) in flight, and the main loop issues
// batch i+1 before it consumes batch i.  The first batch can be issued before
// the query is known (its loads do not depend on it).
constexpr int kAttnU = 4;

// 16 bytes with the streaming hint: the line is not kept in L2 after it has been delivered.
__device__ __forceinline__ uint4 load16_stream(const void* p) {
  typedef unsigned v4u_t __attribute__((ext_vector_type(4)));
  const v4u_t v = __builtin_nontemporal_load(reinterpret_cast<const v4u_t*>(p));
  return make_uint4(v[0], v[1], v[2], v[3]);
}

// STREAM: the rows are read once per launch (decode steps: every (b, h) has its own rows); without it they
// are read again by other queries of the launch (prefill) and should stay in L2.
template <class T, int DH, bool STREAM = false>
__device__ __forceinline__ void attend_issue(const T* __restrict__ K, const T* __restrict__ V, int base, int j0, int j1,
                                             uint4* kraw, uint4* vraw) {
  using R = RowMap<T, DH>;
  constexpr int EPC = R::EPC, LPR = R::LPR, RPL = R::RPL;
  const int lane = threadIdx.x & 63;
  const int sub = lane % LPR, rr = lane / LPR;
#pragma unroll
  for (int u = 0; u < kAttnU; ++u) {
    const int j = base + u * RPL + rr;
    const size_t off = (size_t)(j < j1 ? j : j0) * DH + sub * EPC;      // clamped: no branch around the loads
    if constexpr (STREAM) {
      kraw[u] = load16_stream(K + off);
      vraw[u] = load16_stream(V + off);
    } else {
      kraw[u] = *reinterpret_cast<const uint4*>(K + off);
      vraw[u] = *reinterpret_cast<const uint4*>(V + off);
    }
  }
}

// kraw / vraw: the batch at base = j0, already issued by attend_issue (only if j0 < j1).
template <class T, int DH, bool STREAM = false>
__device__ __forceinline__ void wave_attend(const float* q, const T* __restrict__ K, const T* __restrict__ V,
                                            int j0, int j1, uint4* kraw, uint4* vraw,
                                            float& m_out, float& l_out, float* acc) {
  using R = RowMap<T, DH>;
  constexpr int EPC = R::EPC, LPR = R::LPR, RPL = R::RPL, U = kAttnU;
  const int lane = threadIdx.x & 63;
  const int rr = lane / LPR;
  float m = kNegBig, l = 0.f;
#pragma unroll
  for (int e = 0; e < EPC; ++e) acc[e] = 0.f;

  for (int base = j0; base < j1; base += RPL * U) {
    uint4 knext[U], vnext[U];
    const int nb = base + RPL * U;
    if (nb < j1) attend_issue<T, DH, STREAM>(K, V, nb, j0, j1, knext, vnext);
    float s[U];
    float mx = m;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float kf[EPC];
      Chunk<T>::unpack(kraw[u], kf);
      float dot = 0.f;
#pragma unroll
      for (int e = 0; e < EPC; ++e) dot = fmaf(q[e], kf[e], dot);
#pragma unroll
      for (int o = LPR / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o, kWave);
      s[u] = (base + u * RPL + rr < j1) ? dot : kNegBig;
      mx = fmaxf(mx, s[u]);
    }
    const float scale = __expf(m - mx);
    l *= scale;
#pragma unroll
    for (int e = 0; e < EPC; ++e) acc[e] *= scale;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float p = (base + u * RPL + rr < j1) ? __expf(s[u] - mx) : 0.f;
      float vf[EPC];
      Chunk<T>::unpack(vraw[u], vf);
      l += p;
#pragma unroll
      for (int e = 0; e < EPC; ++e) acc[e] = fmaf(p, vf[e], acc[e]);
    }
    m = mx;
    if (nb < j1) {
#pragma unroll
      for (int u = 0; u < U; ++u) { kraw[u] = knext[u]; vraw[u] = vnext[u]; }
    }
  }
  // merge the RPL slots (lanes that share `sub`)
#pragma unroll
  for (int o = LPR; o < kWave; o <<= 1) {
    const float m2 = __shfl_xor(m, o, kWave);
    const float l2 = __shfl_xor(l, o, kWave);
    const float M = fmaxf(m, m2);
    const float a = __expf(m - M), b = __expf(m2 - M);
    l = l * a + l2 * b;
#pragma unroll
    for (int e = 0; e < EPC; ++e) {
      const float a2 = __shfl_xor(acc[e], o, kWave);
      acc[e] = acc[e] * a + a2 * b;
    }
    m = M;
  }
  m_out = m;
  l_out = l;
}

// ---------------------------------------------------------------------------
// Block decoder, decode step.  Grid: n_split workgroups per (b, h) (+ optional extra
// workgroups that turn the MLP up-projection into its activation).  The
// workgroup first finishes this head's q, k, v (split-K pieces + bias, rotary),
// appends k, v to the cache at slot n_old, then its NW waves split the n_old
// cached rows; partial (m, l, acc) meet in LDS, where the new row joins them.
// With few (b, h) pairs (small batches) one workgroup per pair would leave most
// CUs idle however long the cache is: the rows of a pair are then cut into
// n_split contiguous ranges, one workgroup each; a workgroup leaves its
// unnormalised (acc, m, l) in `split_out` and attn_split_combine_kernel merges
// the ranges in a fixed order.  Range 0 appends the new row and counts it in.
// ---------------------------------------------------------------------------
template <class T, int DH, int NW>
__global__ __launch_bounds__(NW * 64) void attn_block_decode_kernel(PartialSrc qkv, T* __restrict__ Kc, T* __restrict__ Vc,
                                                                    const float2* __restrict__ rope, int rot,
                                                                    T* __restrict__ out, size_t out_lo_off, int n_heads,
                                                                    int n_old_arg, const int* __restrict__ n_dev, int n_cap,
                                                                    int n_attn_blocks, GeluJob gelu, int n_split,
                                                                    float* __restrict__ split_out) {
  using R = RowMap<T, DH>;
  constexpr int EPC = R::EPC, LPR = R::LPR;
  __shared__ float s_m[NW], s_l[NW];
  __shared__ float s_acc[NW][DH];
  __shared__ float s_q[DH], s_k[DH], s_v[DH];
  __shared__ float s_new;
  if ((int)blockIdx.x >= n_attn_blocks) {
    gelu_reduce_block<T>(gelu, blockIdx.x - n_attn_blocks, gridDim.x - n_attn_blocks);
    return;
  }
  // the number of cached blocks may live in device memory, so that a captured graph of the
  // step stays valid while the cache grows
  const int bh = blockIdx.x / n_split, sp = blockIdx.x - bh * n_split;
  const int b = bh / n_heads, h = bh - b * n_heads;
  const int n_old = n_dev ? min(n_dev[b], n_cap - 1) : n_old_arg;
  const int D = n_heads * DH, half = rot / 2;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR;
  T* K = Kc + (size_t)bh * n_cap * DH;
  T* V = Vc + (size_t)bh * n_cap * DH;
  // the cached rows of this workgroup's range and, inside it, of this wave: their first batch of loads
  // goes out before anything else
  const int range = (n_old + n_split - 1) / n_split;
  const int r0 = min(sp * range, n_old), r1 = min(r0 + range, n_old);
  const int per = (r1 - r0 + NW - 1) / NW;
  const int j0 = min(r0 + wave * per, r1), j1 = min(j0 + per, r1);
  uint4 kraw[kAttnU], vraw[kAttnU];
  if (j0 < j1) attend_issue<T, DH, true>(K, V, j0, j0, j1, kraw, vraw);

  // q, k, v of this head: sum the pieces, rotate q and k at position n_old, append k and v
  const int d = threadIdx.x;
  float2 cs = make_float2(1.f, 0.f);
  if (d < rot) cs = rope[(size_t)n_old * half + (d < half ? d : d - half)];
  if (d < DH) {
    const size_t base = (size_t)b * 3 * D + h * DH + d;
    s_q[d] = partial_value(qkv, base, h * DH + d);
    s_k[d] = partial_value(qkv, base + D, D + h * DH + d);
    s_v[d] = partial_value(qkv, base + 2 * D, 2 * D + h * DH + d);
  }
  __syncthreads();
  float qd = 0.f, kd = 0.f;
  if (d < DH) {
    qd = s_q[d];
    kd = s_k[d];
    if (d < rot) {
      if (d < half) { qd = qd * cs.x - s_q[d + half] * cs.y; kd = kd * cs.x - s_k[d + half] * cs.y; }
      else          { qd = qd * cs.x + s_q[d - half] * cs.y; kd = kd * cs.x + s_k[d - half] * cs.y; }
    }
  }
  __syncthreads();
  if (d < DH) {
    const T kt = from_float<T>(kd), vt = from_float<T>(s_v[d]);
    if (sp == 0) {
      K[(size_t)n_old * DH + d] = kt;
      V[(size_t)n_old * DH + d] = vt;
    }
    s_q[d] = qd * rsqrtf((float)DH);
    s_k[d] = to_float<T>(kt);          // the new row takes part with its stored (rounded) values
    s_v[d] = to_float<T>(vt);
  }
  __syncthreads();
  if (wave == 0) {
    float dot = 0.f;
    for (int e = lane; e < DH; e += 64) dot = fmaf(s_q[e], s_k[e], dot);
    dot = wave_sum(dot);
    if (lane == 0) s_new = dot;
  }
  float q[EPC];
#pragma unroll
  for (int e = 0; e < EPC; ++e) q[e] = s_q[sub * EPC + e];

  float m, l, acc[EPC];
  wave_attend<T, DH, true>(q, K, V, j0, j1, kraw, vraw, m, l, acc);
  if (lane < LPR) {
    if (lane == 0) { s_m[wave] = m; s_l[wave] = l; }
#pragma unroll
    for (int e = 0; e < EPC; ++e) s_acc[wave][sub * EPC + e] = acc[e];
  }
  __syncthreads();
  const float snew = sp == 0 ? s_new : kNegBig;          // the new row belongs to range 0
  for (int dd = threadIdx.x; dd < DH; dd += NW * 64) {
    float M = snew;
#pragma unroll
    for (int w = 0; w < NW; ++w) M = fmaxf(M, s_m[w]);
    const float fn = sp == 0 ? __expf(snew - M) : 0.f;
    float L = fn, o = fn * s_v[dd];
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float f = __expf(s_m[w] - M);
      L += s_l[w] * f;
      o += s_acc[w][dd] * f;
    }
    if (n_split == 1) {
      store_act<T>(out, (size_t)b * D + h * DH + dd, out_lo_off, o / L);
    } else {
      float* po = split_out + (size_t)blockIdx.x * (DH + 2);
      po[dd] = o;
      if (dd == 0) { po[DH] = M; po[DH + 1] = L; }
    }
  }
}

// Merge of the n_split ranges of every (b, h): one wave per pair, ranges in index order.
template <class T, int DH>
__global__ __launch_bounds__(256) void attn_split_combine_kernel(const float* __restrict__ split_out, int n_split, int n_pairs,
                                                                 int n_heads, T* __restrict__ out, size_t out_lo_off) {
  const int lane = threadIdx.x & 63;
  const int bh = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (bh >= n_pairs) return;
  const int b = bh / n_heads, h = bh - b * n_heads, D = n_heads * DH;
  const float* p = split_out + (size_t)bh * n_split * (DH + 2);
  float M = kNegBig;
  for (int s = 0; s < n_split; ++s) M = fmaxf(M, p[(size_t)s * (DH + 2) + DH]);
  float L = 0.f, o[(DH + 63) / 64];
#pragma unroll
  for (int c = 0; c < (DH + 63) / 64; ++c) o[c] = 0.f;
  for (int s = 0; s < n_split; ++s) {
    const float* ps = p + (size_t)s * (DH + 2);
    const float f = __expf(ps[DH] - M);
    L += ps[DH + 1] * f;
#pragma unroll
    for (int c = 0; c < (DH + 63) / 64; ++c) {
      const int d = lane + 64 * c;
      if (d < DH) o[c] += ps[d] * f;
    }
  }
#pragma unroll
  for (int c = 0; c < (DH + 63) / 64; ++c) {
    const int d = lane + 64 * c;
    if (d < DH) store_act<T>(out, (size_t)b * D + h * DH + d, out_lo_off, o[c] / L);
  }
}

// ---------------------------------------------------------------------------
// Block decoder, prefill: one wave per query, query i attends rows [0, i].
// ---------------------------------------------------------------------------
template <class T, int DH>
__global__ __launch_bounds__(256) void attn_block_prefill_kernel(const float* __restrict__ qkv, const T* __restrict__ Kc,
                                                                 const T* __restrict__ Vc, T* __restrict__ out,
                                                                 size_t out_lo_off, int n_heads, int n_q, int n_cap) {
  using R = RowMap<T, DH>;
  constexpr int EPC = R::EPC, LPR = R::LPR;
  const int bh = blockIdx.x;
  const int b = bh / n_heads, h = bh - b * n_heads;
  const int D = n_heads * DH;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i = n_q - 1 - (blockIdx.y * 4 + wave);      // long rows first
  if (i < 0) return;
  const int sub = lane % LPR;
  const size_t row = (size_t)b * n_q + i;
  const float sc = rsqrtf((float)DH);
  float q[EPC];
  const float* qp = qkv + row * 3 * D + h * DH + sub * EPC;
#pragma unroll
  for (int e = 0; e < EPC; ++e) q[e] = qp[e] * sc;
  const T* K = Kc + (size_t)bh * n_cap * DH;
  const T* V = Vc + (size_t)bh * n_cap * DH;
  float m, l, acc[EPC];
  uint4 kraw[kAttnU], vraw[kAttnU];
  attend_issue<T, DH>(K, V, 0, 0, i + 1, kraw, vraw);
  wave_attend<T, DH>(q, K, V, 0, i + 1, kraw, vraw, m, l, acc);
  if (lane < LPR) {
    const float inv = 1.0f / l;
    float o[EPC];
#pragma unroll
    for (int e = 0; e < EPC; ++e) o[e] = acc[e] * inv;
    T* dst = out + row * D + h * DH + sub * EPC;
    const uint4 hi = Chunk<T>::pack(o);
    *reinterpret_cast<uint4*>(dst) = hi;
    if (out_lo_off) {
      float back[EPC];
      Chunk<T>::unpack(hi, back);
#pragma unroll
      for (int e = 0; e < EPC; ++e) o[e] -= back[e];
      *reinterpret_cast<uint4*>(dst + out_lo_off) = Chunk<T>::pack(o);
    }
  }
}

// ---------------------------------------------------------------------------
// Block decoder, prefill, bf16 mode with many queries: causal attention as two
// dense contractions on the matrix cores (v_mfma_f32_16x16x32_bf16).
// Workgroup = one (b, h) x 64 consecutive queries, wave = 16 of them.  Keys are
// walked in blocks of 32 up to the diagonal:
//   S = Q K^T   A operand = q (scaled by 1/sqrt(d_h), split into bf16 hi + remainder,
//               two MFMAs), B operand = a K row chunk straight from the cache;
//   online softmax on S in the MFMA result layout (a lane holds 4 queries x 1 key per
//               16-key tile; row max / sum by shuffles over the 16 lanes of a row);
//   O += P V    P goes through LDS to become an A operand (hi + remainder again), V is
//               staged transposed in LDS ([d][key]) so that a B fragment (8 consecutive
//               keys of one d) is one 16-byte read.
// Results match the plain kernel to fp32 rounding: every bf16 operand is either an exact
// stored value (K, V) or carried as hi + remainder (q, p).
// ---------------------------------------------------------------------------
typedef __bf16 abf16x8_t __attribute__((ext_vector_type(8)));
typedef float af32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void split8(const float* x, abf16x8_t& hi, abf16x8_t& lo) {
  uint32_t h[4], l[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const uint32_t h0 = float_to_bf16_bits(x[2 * e]), h1 = float_to_bf16_bits(x[2 * e + 1]);
    const uint32_t l0 = float_to_bf16_bits(x[2 * e] - bf16_bits_to_float(h0));
    const uint32_t l1 = float_to_bf16_bits(x[2 * e + 1] - bf16_bits_to_float(h1));
    h[e] = h0 | (h1 << 16);
    l[e] = l0 | (l1 << 16);
  }
  hi = __builtin_bit_cast(abf16x8_t, make_uint4(h[0], h[1], h[2], h[3]));
  lo = __builtin_bit_cast(abf16x8_t, make_uint4(l[0], l[1], l[2], l[3]));
}

template <int DH>
__global__ __launch_bounds__(256) void attn_block_prefill_mfma_kernel(const float* __restrict__ qkv, const bf16_t* __restrict__ Kc,
                                                                      const bf16_t* __restrict__ Vc, bf16_t* __restrict__ out,
                                                                      size_t out_lo_off, int n_heads, int n_q, int n_cap) {
  constexpr int KB = 32;                 // keys per block
  constexpr int KP = KB + 8;             // padded key stride of the LDS tiles (elements)
  constexpr int NC = DH / 32;            // 32-dim chunks of a head
  constexpr int ND = DH / 16;            // 16-dim tiles of the output
  __shared__ __attribute__((aligned(16))) uint16_t sVt[DH * KP];          // V block, transposed: [d][key]
  __shared__ __attribute__((aligned(16))) uint16_t sP[4][2][16 * KP];     // per wave: p hi / remainder, [query][key]

  const int bh = blockIdx.y;
  const int b = bh / n_heads, h = bh - b * n_heads;
  const int D = n_heads * DH;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 15, lg = lane >> 4;
  const int n_tiles = (n_q + 63) / 64;
  const int q_wg = (n_tiles - 1 - (int)blockIdx.x) * 64;      // long rows first
  const int q_w = q_wg + wave * 16;                           // first query of this wave
  const bf16_t* K = Kc + (size_t)bh * n_cap * DH;
  const bf16_t* V = Vc + (size_t)bh * n_cap * DH;

  // A operand: q of query q_w + lr, dims 32 c + 8 lg .. + 8, scaled, as hi + remainder
  abf16x8_t qh[NC], ql[NC];
  {
    const int qi = min(q_w + lr, n_q - 1);
    const float* qp = qkv + ((size_t)b * n_q + qi) * 3 * D + h * DH + lg * 8;
    const float sc = rsqrtf((float)DH);
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const float4 a = *reinterpret_cast<const float4*>(qp + c * 32), bq = *reinterpret_cast<const float4*>(qp + c * 32 + 4);
      const float x[8] = {a.x * sc, a.y * sc, a.z * sc, a.w * sc, bq.x * sc, bq.y * sc, bq.z * sc, bq.w * sc};
      split8(x, qh[c], ql[c]);
    }
  }
  af32x4_t o[ND];
#pragma unroll
  for (int t = 0; t < ND; ++t) o[t] = af32x4_t{0.f, 0.f, 0.f, 0.f};
  float m[4], l[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) { m[r] = kNegBig; l[r] = 0.f; }

  const int last_key_wg = min(q_wg + 63, n_q - 1);
  const int last_key_w = min(q_w + 15, n_q - 1);
  // The V chunks and K fragments of a key block travel in registers while the block before it is
  // worked on: thread t stages V of key c / (DH/8), dims 8 (c % (DH/8)) .. + 8 for its chunks c = t, t + 256;
  // a lane's K fragments are rows k0 + 16 t + lr, dims 32 c + 8 lg .. + 8.
  constexpr int VCH = (KB * (DH / 8) + 255) / 256;
  uint4 vnext[VCH], knext[2][NC];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int u = 0; u < VCH; ++u) {
      const int c = min(tid + u * 256, KB * (DH / 8) - 1);
      const int key = c / (DH / 8), dc = c - key * (DH / 8);
      vnext[u] = *reinterpret_cast<const uint4*>(V + (size_t)min(k0 + key, n_cap - 1) * DH + dc * 8);
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const bf16_t* kp = K + (size_t)min(k0 + t * 16 + lr, n_cap - 1) * DH + lg * 8;
#pragma unroll
      for (int c = 0; c < NC; ++c) knext[t][c] = *reinterpret_cast<const uint4*>(kp + c * 32);
    }
  };
  fetch(0);
  for (int k0 = 0; k0 <= last_key_wg; k0 += KB) {
    // V block -> LDS, transposed
    __syncthreads();                       // the previous block's fragments have been read
#pragma unroll
    for (int u = 0; u < VCH; ++u) {
      const int c = tid + u * 256;
      if (c < KB * (DH / 8)) {
        const int key = c / (DH / 8), dc = c - key * (DH / 8);
        uint4 v = vnext[u];
        if (k0 + key >= n_q) v = make_uint4(0u, 0u, 0u, 0u);     // never-written rows may hold NaN patterns: 0 * NaN
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) sVt[(dc * 8 + e) * KP + key] = (uint16_t)(w[e >> 1] >> ((e & 1) * 16));
      }
    }
    abf16x8_t kcur[2][NC];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int c = 0; c < NC; ++c) kcur[t][c] = __builtin_bit_cast(abf16x8_t, knext[t][c]);
    if (k0 + KB <= last_key_wg) fetch(k0 + KB);          // uniform over the workgroup: the next block starts its trip
    __syncthreads();
    if (k0 <= last_key_w) {                // blocks entirely above this wave's diagonal contribute nothing
      // S = Q K^T for two 16-key tiles
      af32x4_t sacc[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        sacc[t] = af32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < NC; ++c) {
          const abf16x8_t kf = kcur[t][c];
          sacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qh[c], kf, sacc[t], 0, 0, 0);
          sacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ql[c], kf, sacc[t], 0, 0, 0);
        }
      }
      // lane holds S[query q_w + 4 lg + r][key k0 + 16 t + lr]
      float alpha[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int qi = q_w + 4 * lg + r;
        float s0 = (k0 + lr <= qi) ? sacc[0][r] : kNegBig;
        float s1 = (k0 + 16 + lr <= qi) ? sacc[1][r] : kNegBig;
        const float mx = row16_max(fmaxf(s0, s1));        // over the 16 lanes that hold this query's keys
        const float mn = fmaxf(m[r], mx);
        const float p0 = (k0 + lr <= qi) ? __expf(s0 - mn) : 0.f;
        const float p1 = (k0 + 16 + lr <= qi) ? __expf(s1 - mn) : 0.f;
        const float ps = row16_sum(p0 + p1);
        alpha[r] = __expf(m[r] - mn);
        l[r] = l[r] * alpha[r] + ps;
        m[r] = mn;
        // p -> LDS as hi + remainder, [query][key]
        const uint16_t h0 = float_to_bf16_bits(p0), h1 = float_to_bf16_bits(p1);
        sP[wave][0][(4 * lg + r) * KP + lr] = h0;
        sP[wave][0][(4 * lg + r) * KP + 16 + lr] = h1;
        sP[wave][1][(4 * lg + r) * KP + lr] = float_to_bf16_bits(p0 - bf16_bits_to_float(h0));
        sP[wave][1][(4 * lg + r) * KP + 16 + lr] = float_to_bf16_bits(p1 - bf16_bits_to_float(h1));
      }
#pragma unroll
      for (int t = 0; t < ND; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) o[t][r] *= alpha[r];
      __builtin_amdgcn_wave_barrier();
      // O += P V: A = p of query q_w + lr, keys 8 lg .. + 8; B = V^T rows d = 16 t + lr, the same keys
      const abf16x8_t ph = __builtin_bit_cast(abf16x8_t, *reinterpret_cast<const uint4*>(&sP[wave][0][lr * KP + lg * 8]));
      const abf16x8_t pl = __builtin_bit_cast(abf16x8_t, *reinterpret_cast<const uint4*>(&sP[wave][1][lr * KP + lg * 8]));
#pragma unroll
      for (int t = 0; t < ND; ++t) {
        const abf16x8_t vf = __builtin_bit_cast(abf16x8_t, *reinterpret_cast<const uint4*>(&sVt[(t * 16 + lr) * KP + lg * 8]));
        o[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ph, vf, o[t], 0, 0, 0);
        o[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pl, vf, o[t], 0, 0, 0);
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
  // lane holds O[query q_w + 4 lg + r][d = 16 t + lr]
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int qi = q_w + 4 * lg + r;
    if (qi < n_q) {
      const float inv = 1.0f / l[r];
      const size_t row = (size_t)b * n_q + qi;
#pragma unroll
      for (int t = 0; t < ND; ++t) store_act<bf16_t>(out, row * D + h * DH + t * 16 + lr, out_lo_off, o[t][r] * inv);
    }
  }
}

// ---------------------------------------------------------------------------
// Block decoder: rotary on q (in place) and k, append k, v to the block cache.
// One workgroup per row.
// ---------------------------------------------------------------------------
template <class T>
__global__ __launch_bounds__(256) void rope_append_kernel(PartialSrc src, T* __restrict__ Kc, T* __restrict__ Vc,
                                                          const float2* __restrict__ rope, int n_new, int pos0,
                                                          int n_heads, int DH, int rot,
                                                          int n_cap, int n_rows, GeluJob gelu) {
  if ((int)blockIdx.x >= n_rows) {
    gelu_reduce_block<T>(gelu, blockIdx.x - n_rows, gridDim.x - n_rows);
    return;
  }
  const int m = blockIdx.x;
  const int b = m / n_new, pos = pos0 + (m - b * n_new);
  const int D = n_heads * DH, half = rot / 2;
  const size_t rbase = (size_t)m * 3 * D;
  float* q = const_cast<float*>(src.base) + rbase;      // plane 0 receives the finished q
  const bool pieces = src.splits > 1 || src.bias != nullptr;
  for (int idx = threadIdx.x; idx < n_heads * half; idx += blockDim.x) {
    const int h = idx / half, t = idx - h * half;
    const float2 cs = rope[(size_t)pos * half + t];
    const int d0 = h * DH + t, d1 = d0 + half;
    const float q0 = partial_value(src, rbase + d0, d0), q1 = partial_value(src, rbase + d1, d1);
    q[d0] = q0 * cs.x - q1 * cs.y;
    q[d1] = q1 * cs.x + q0 * cs.y;
    const float k0 = partial_value(src, rbase + D + d0, D + d0), k1 = partial_value(src, rbase + D + d1, D + d1);
    const size_t base = ((size_t)(b * n_heads + h) * n_cap + pos) * DH;
    Kc[base + t] = from_float<T>(k0 * cs.x - k1 * cs.y);
    Kc[base + t + half] = from_float<T>(k1 * cs.x + k0 * cs.y);
  }
  for (int idx = threadIdx.x; idx < D; idx += blockDim.x) {
    const int h = idx / DH, d = idx - h * DH;
    const size_t base = ((size_t)(b * n_heads + h) * n_cap + pos) * DH;
    if (d >= rot) {
      Kc[base + d] = from_float<T>(partial_value(src, rbase + D + idx, D + idx));
      if (pieces) q[idx] = partial_value(src, rbase + idx, idx);
    }
    Vc[base + d] = from_float<T>(partial_value(src, rbase + 2 * D + idx, 2 * D + idx));
  }
}

// ---------------------------------------------------------------------------
// Token decoder local attention.  One wave per (b, h); the local K, V of the
// pair (<= l_cap rows) are staged in LDS as floats of the stored values.
// LDS per wave: K [l_cap][DH], V [l_cap][DH], raw q [DH], raw k [DH].
// ---------------------------------------------------------------------------
template <class T, int DH>
__global__ void attn_local_kernel(PartialSrc qkv, T* __restrict__ Kl, T* __restrict__ Vl,
                                  const float2* __restrict__ rope, T* __restrict__ out, size_t out_lo_off,
                                  int n_pairs, int n_heads, int rot, int rows, int pos0, int l_cap,
                                  int n_attn_blocks, GeluJob gelu) {
  extern __shared__ float smem[];
  if ((int)blockIdx.x >= n_attn_blocks) {
    gelu_reduce_block<T>(gelu, blockIdx.x - n_attn_blocks, gridDim.x - n_attn_blocks);
    return;
  }
  constexpr int DPL = (DH + 63) / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nw = blockDim.x >> 6;
  const int pair_raw = blockIdx.x * nw + wave;
  const bool active = pair_raw < n_pairs;
  const int pair = active ? pair_raw : n_pairs - 1;     // idle waves shadow a valid pair, write nothing
  const int b = pair / n_heads, h = pair - b * n_heads;
  const int D = n_heads * DH, half = rot / 2;
  float* sK = smem + (size_t)wave * (2 * l_cap + 2) * DH;
  float* sV = sK + l_cap * DH;
  float* sq = sV + l_cap * DH;
  float* sk = sq + DH;
  T* Kg = Kl + (size_t)pair * l_cap * DH;
  T* Vg = Vl + (size_t)pair * l_cap * DH;
  const float sc = rsqrtf((float)DH);

  for (int idx = lane; idx < pos0 * DH; idx += 64) {
    sK[idx] = to_float<T>(Kg[idx]);
    sV[idx] = to_float<T>(Vg[idx]);
  }
  for (int i = 0; i < rows; ++i) {
    const int pos = pos0 + i;
    const size_t row = (size_t)b * rows + i;
    const size_t src = row * 3 * D + h * DH;
    float vv[DPL];
#pragma unroll
    for (int c = 0; c < DPL; ++c) {
      const int d = lane + 64 * c;
      if (d < DH) {
        sq[d] = partial_value(qkv, src + d, h * DH + d);
        sk[d] = partial_value(qkv, src + D + d, D + h * DH + d);
        vv[c] = partial_value(qkv, src + 2 * D + d, 2 * D + h * DH + d);
      }
    }
    __syncthreads();
    float qv[DPL];
#pragma unroll
    for (int c = 0; c < DPL; ++c) {
      const int d = lane + 64 * c;
      if (d < DH) {
        float qd = sq[d], kd = sk[d];
        if (d < rot) {
          const int t = d < half ? d : d - half;
          const float2 cs = rope[(size_t)pos * half + t];
          if (d < half) { qd = qd * cs.x - sq[d + half] * cs.y; kd = kd * cs.x - sk[d + half] * cs.y; }
          else          { qd = qd * cs.x + sq[d - half] * cs.y; kd = kd * cs.x + sk[d - half] * cs.y; }
        }
        qv[c] = qd * sc;
        const T kt = from_float<T>(kd), vt = from_float<T>(vv[c]);
        sK[pos * DH + d] = to_float<T>(kt);
        sV[pos * DH + d] = to_float<T>(vt);
        if (active) { Kg[pos * DH + d] = kt; Vg[pos * DH + d] = vt; }
      } else {
        qv[c] = 0.f;
      }
    }
    __syncthreads();
    float m = kNegBig, l = 0.f, acc[DPL];
#pragma unroll
    for (int c = 0; c < DPL; ++c) acc[c] = 0.f;
    for (int j = 0; j <= pos; ++j) {
      float dot = 0.f;
#pragma unroll
      for (int c = 0; c < DPL; ++c) {
        const int d = lane + 64 * c;
        if (d < DH) dot = fmaf(qv[c], sK[j * DH + d], dot);
      }
      dot = wave_sum(dot);
      const float mx = fmaxf(m, dot);
      const float scale = __expf(m - mx), p = __expf(dot - mx);
      l = l * scale + p;
#pragma unroll
      for (int c = 0; c < DPL; ++c) {
        const int d = lane + 64 * c;
        if (d < DH) acc[c] = acc[c] * scale + p * sV[j * DH + d];
      }
      m = mx;
    }
    if (active) {
#pragma unroll
      for (int c = 0; c < DPL; ++c) {
        const int d = lane + 64 * c;
        if (d < DH) store_act<T>(out, row * D + h * DH + d, out_lo_off, acc[c] / l);
      }
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------
// Token decoder local attention with at most MAXJ keys per query (the usual case:
// prefix tokens + block length is small).  One wave per (b, h), everything in
// registers: lane owns dims d = lane + 64 c of q, of the new k, v and of every
// cached row, so scores are lane-local products plus one wave reduction, and the
// rotary partner comes from a shuffle.  All global loads of a row (cached rows,
// the split-K pieces of q, k, v, the rotary pair) are issued before the first use:
// one trip to memory per launch.  Same arithmetic as attn_local_kernel except
// that the softmax is taken over all scores at once instead of online.
// ---------------------------------------------------------------------------
template <int DPL>
__device__ __forceinline__ float shuffle_dim(const float* x, int p) {      // element p of a vector spread as x[c] = dim lane + 64 c
  float r = 0.f;
#pragma unroll
  for (int c = 0; c < DPL; ++c) {
    const float t = __shfl(x[c], p & 63, kWave);
    if ((p >> 6) == c) r = t;
  }
  return r;
}

template <class T, int DH, int MAXJ>
__global__ __launch_bounds__(256) void attn_local_reg_kernel(PartialSrc qkv, T* __restrict__ Kl, T* __restrict__ Vl,
                                                             const float2* __restrict__ rope, T* __restrict__ out,
                                                             size_t out_lo_off, int n_pairs, int n_heads, int rot, int rows,
                                                             int pos0, int l_cap, int n_attn_blocks, GeluJob gelu) {
  if ((int)blockIdx.x >= n_attn_blocks) {
    gelu_reduce_block<T>(gelu, blockIdx.x - n_attn_blocks, gridDim.x - n_attn_blocks);
    return;
  }
  constexpr int DPL = (DH + 63) / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int pair_raw = blockIdx.x * (blockDim.x >> 6) + wave;
  const bool active = pair_raw < n_pairs;
  const int pair = active ? pair_raw : n_pairs - 1;     // idle waves shadow a valid pair, write nothing
  const int b = pair / n_heads, h = pair - b * n_heads;
  const int D = n_heads * DH, half = rot / 2;
  T* Kg = Kl + (size_t)pair * l_cap * DH;
  T* Vg = Vl + (size_t)pair * l_cap * DH;
  const float sc = rsqrtf((float)DH);
  int dcl[DPL];
#pragma unroll
  for (int c = 0; c < DPL; ++c) dcl[c] = min(lane + 64 * c, DH - 1);        // clamped dim: loads need no branch

  // cached rows [0, pos0); slots past pos0 are zero until a new row lands there
  float Kr[MAXJ][DPL], Vr[MAXJ][DPL];
#pragma unroll
  for (int j = 0; j < MAXJ; ++j) {
    const int jc = min(j, max(pos0 - 1, 0));
#pragma unroll
    for (int c = 0; c < DPL; ++c) {
      const float kx = to_float<T>(Kg[jc * DH + dcl[c]]), vx = to_float<T>(Vg[jc * DH + dcl[c]]);
      Kr[j][c] = j < pos0 ? kx : 0.f;          // never-written cache memory may hold NaN patterns
      Vr[j][c] = j < pos0 ? vx : 0.f;
    }
  }
  for (int i = 0; i < rows; ++i) {
    const int pos = pos0 + i;
    const size_t row = (size_t)b * rows + i;
    float q[DPL], k[DPL], v[DPL];
    float2 cs[DPL];
#pragma unroll
    for (int c = 0; c < DPL; ++c) {
      const int d = dcl[c];
      const size_t src = row * 3 * D + h * DH + d;
      q[c] = qkv.bias ? qkv.bias[h * DH + d] : 0.f;
      k[c] = qkv.bias ? qkv.bias[D + h * DH + d] : 0.f;
      v[c] = qkv.bias ? qkv.bias[2 * D + h * DH + d] : 0.f;
      cs[c] = rope[(size_t)pos * half + (d < rot ? (d < half ? d : d - half) : 0)];
      for (int s0 = 0; s0 < qkv.splits; s0 += 4) {
        float t[3][4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const float* pb = qkv.base + (size_t)min(s0 + u, qkv.splits - 1) * qkv.stride + src;
          t[0][u] = pb[0]; t[1][u] = pb[D]; t[2][u] = pb[2 * D];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const float m = s0 + u < qkv.splits ? 1.f : 0.f;
          q[c] += m * t[0][u]; k[c] += m * t[1][u]; v[c] += m * t[2][u];
        }
      }
    }
    float qv[DPL];
#pragma unroll
    for (int c = 0; c < DPL; ++c) {
      const int d = lane + 64 * c;
      float qd = q[c], kd = k[c];
      const int partner = d < half ? d + half : d - half;
      const float qp = shuffle_dim<DPL>(q, partner & (64 * DPL - 1)), kp = shuffle_dim<DPL>(k, partner & (64 * DPL - 1));
      if (d < rot) {
        if (d < half) { qd = qd * cs[c].x - qp * cs[c].y; kd = kd * cs[c].x - kp * cs[c].y; }
        else          { qd = qd * cs[c].x + qp * cs[c].y; kd = kd * cs[c].x + kp * cs[c].y; }
      }
      qv[c] = d < DH ? qd * sc : 0.f;
      const T kt = from_float<T>(kd), vt = from_float<T>(v[c]);
      if (active && d < DH) { Kg[pos * DH + d] = kt; Vg[pos * DH + d] = vt; }
      const float kf = to_float<T>(kt), vf = to_float<T>(vt);
#pragma unroll
      for (int j = 0; j < MAXJ; ++j)
        if (j == pos) { Kr[j][c] = kf; Vr[j][c] = vf; }
    }
    float sj[MAXJ], m = kNegBig;
#pragma unroll
    for (int j = 0; j < MAXJ; ++j) {
      float dot = 0.f;
#pragma unroll
      for (int c = 0; c < DPL; ++c) dot = fmaf(qv[c], Kr[j][c], dot);
      dot = wave_sum(dot);
      sj[j] = j <= pos ? dot : kNegBig;
      m = fmaxf(m, sj[j]);
    }
    float l = 0.f, acc[DPL];
#pragma unroll
    for (int c = 0; c < DPL; ++c) acc[c] = 0.f;
#pragma unroll
    for (int j = 0; j < MAXJ; ++j) {
      const float pj = j <= pos ? __expf(sj[j] - m) : 0.f;
      l += pj;
#pragma unroll
      for (int c = 0; c < DPL; ++c) acc[c] = fmaf(pj, Vr[j][c], acc[c]);
    }
    if (active) {
#pragma unroll
      for (int c = 0; c < DPL; ++c) {
        const int d = lane + 64 * c;
        if (d < DH) store_act<T>(out, row * D + h * DH + d, out_lo_off, acc[c] / l);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
#define BT_DISPATCH_DH(DHV, ...)                         \
  switch (DHV) {                                         \
    case 32:  { constexpr int DH = 32;  __VA_ARGS__; break; }  \
    case 64:  { constexpr int DH = 64;  __VA_ARGS__; break; }  \
    case 128: { constexpr int DH = 128; __VA_ARGS__; break; }  \
    default: return hipErrorInvalidValue;                \
  }

hipError_t launch_rope_append(int dtype, const PartialSrc& src, void* Kc, void* Vc, const float2* rope,
                              int n_rows, int n_new, int pos0, int n_heads, int d_head, int rot,
                              int n_cap, const GeluJob& gelu, hipStream_t s) {
  if (n_rows <= 0) return hipSuccess;
  if (gelu.rows > 0 && gelu.cols % 4) return hipErrorInvalidValue;
  const int grid = n_rows + gelu_blocks(gelu);
  if (dtype == BT_F32)
    rope_append_kernel<float><<<grid, 256, 0, s>>>(src, (float*)Kc, (float*)Vc, rope, n_new, pos0, n_heads, d_head, rot, n_cap, n_rows, gelu);
  else
    rope_append_kernel<bf16_t><<<grid, 256, 0, s>>>(src, (bf16_t*)Kc, (bf16_t*)Vc, rope, n_new, pos0, n_heads, d_head, rot, n_cap, n_rows, gelu);
  return hipGetLastError();
}

hipError_t launch_gelu_reduce(int dtype, const GeluJob& job, hipStream_t s) {
  const int nb = gelu_blocks(job);
  if (nb == 0) return hipSuccess;
  if (job.cols % 4) return hipErrorInvalidValue;
  if (dtype == BT_F32) gelu_reduce_kernel<float><<<nb, 256, 0, s>>>(job);
  else gelu_reduce_kernel<bf16_t><<<nb, 256, 0, s>>>(job);
  return hipGetLastError();
}

hipError_t launch_attn_block_decode(int dtype, const PartialSrc& qkv, void* Kc, void* Vc, const float2* rope, int rot,
                                    void* out, size_t out_lo_off, int batch, int n_heads, int d_head, int n_old,
                                    const int* n_dev, int n_cap, const GeluJob& gelu, int n_split, float* split_buf,
                                    hipStream_t s) {
  if (!n_dev && (n_old < 0 || n_old >= n_cap)) return hipErrorInvalidValue;
  if (gelu.rows > 0 && gelu.cols % 4) return hipErrorInvalidValue;
  if (n_split < 1 || (n_split > 1 && !split_buf)) return hipErrorInvalidValue;
  const int n_pairs = batch * n_heads;
  const int n_attn = n_pairs * n_split;
  // Waves per workgroup.  Four waves share the rows of a (b, h) when there are few pairs (the chip wants some
  // thousand waves with loads in flight) or when a pair's rows are many bytes; with many pairs of short caches
  // two waves do better (fewer partial results to merge, longer streams per wave).  Per launch at NW = 4 -> 2:
  // cfg3 (2048 pairs, up to 272 rows) 26.7 -> 23.4 us, cfg1's model at batch 256 34.0 -> 28.3, cfg1 17.5 -> 17.3;
  // but cfg2 (384 pairs) 17.2 -> 17.8 and cfg4 (4096 pairs, 1024 rows of 256 bytes) 193.6 -> 200.1.
  const size_t pair_bytes = (size_t)n_cap * d_head * (dtype == BT_F32 ? 4 : 2) * 2;
  const bool two_waves = n_attn >= 768 && pair_bytes <= (192u << 10);
  const int grid = n_attn + gelu_blocks(gelu) * (two_waves ? 2 : 1);      // the GELU workgroups are sized for 256 threads
#define BT_LAUNCH_ATTN_BLOCK_DECODE(T, NWV)                                                                          \
  BT_DISPATCH_DH(d_head, (attn_block_decode_kernel<T, DH, NWV><<<grid, NWV * 64, 0, s>>>(                             \
      qkv, (T*)Kc, (T*)Vc, rope, rot, (T*)out, lo_off, n_heads, n_old, n_dev, n_cap, n_attn, gelu, n_split, split_buf)))
  if (dtype == BT_F32) {
    const size_t lo_off = 0;
    if (two_waves) { BT_LAUNCH_ATTN_BLOCK_DECODE(float, 2); } else { BT_LAUNCH_ATTN_BLOCK_DECODE(float, 4); }
    if (n_split > 1)
      BT_DISPATCH_DH(d_head, (attn_split_combine_kernel<float, DH><<<(n_pairs + 3) / 4, 256, 0, s>>>(
          split_buf, n_split, n_pairs, n_heads, (float*)out, 0)));
  } else {
    const size_t lo_off = out_lo_off;
    if (two_waves) { BT_LAUNCH_ATTN_BLOCK_DECODE(bf16_t, 2); } else { BT_LAUNCH_ATTN_BLOCK_DECODE(bf16_t, 4); }
    if (n_split > 1)
      BT_DISPATCH_DH(d_head, (attn_split_combine_kernel<bf16_t, DH><<<(n_pairs + 3) / 4, 256, 0, s>>>(
          split_buf, n_split, n_pairs, n_heads, (bf16_t*)out, out_lo_off)));
  }
#undef BT_LAUNCH_ATTN_BLOCK_DECODE
  return hipGetLastError();
}

int attn_block_decode_splits(int batch, int n_heads, int n_cap) {
  const int pairs = batch * n_heads;
  if (pairs >= 256) return 1;                       // enough workgroups already
  int s = 512 / pairs;                              // about two workgroups per CU
  const int by_len = n_cap / 128 > 1 ? n_cap / 128 : 1;      // at least 128 cached rows per range at full cache
  if (s > by_len) s = by_len;
  return s > 16 ? 16 : (s < 1 ? 1 : s);
}

hipError_t launch_attn_block_prefill(int dtype, const float* qkv, const void* Kc, const void* Vc,
                                     void* out, size_t out_lo_off, int batch, int n_heads, int d_head, int n_q,
                                     int n_cap, hipStream_t s) {
  if (n_q < 1 || n_q > n_cap) return hipErrorInvalidValue;
  const dim3 grid(batch * n_heads, (n_q + 3) / 4);
  if (dtype == BT_F32) {
    BT_DISPATCH_DH(d_head, (attn_block_prefill_kernel<float, DH><<<grid, 256, 0, s>>>(
        qkv, (const float*)Kc, (const float*)Vc, (float*)out, 0, n_heads, n_q, n_cap)));
  } else if (n_q >= 64) {
    // many queries per sequence: dense contractions on the matrix cores
    const dim3 grid_m((n_q + 63) / 64, batch * n_heads);
    BT_DISPATCH_DH(d_head, (attn_block_prefill_mfma_kernel<DH><<<grid_m, 256, 0, s>>>(
        qkv, (const bf16_t*)Kc, (const bf16_t*)Vc, (bf16_t*)out, out_lo_off, n_heads, n_q, n_cap)));
  } else {
    BT_DISPATCH_DH(d_head, (attn_block_prefill_kernel<bf16_t, DH><<<grid, 256, 0, s>>>(
        qkv, (const bf16_t*)Kc, (const bf16_t*)Vc, (bf16_t*)out, out_lo_off, n_heads, n_q, n_cap)));
  }
  return hipGetLastError();
}

hipError_t launch_attn_local(int dtype, const PartialSrc& qkv, void* Kl, void* Vl, const float2* rope,
                             void* out, size_t out_lo_off, int batch, int n_heads, int d_head, int rot, int rows,
                             int pos0, int l_cap, const GeluJob& gelu, hipStream_t s) {
  if (rows < 1 || pos0 < 0 || pos0 + rows > l_cap) return hipErrorInvalidValue;
  if (gelu.rows > 0 && gelu.cols % 4) return hipErrorInvalidValue;
  const int n_pairs = batch * n_heads;
  // few keys (the usual case): register kernel, sized by the number of keys this launch can see
  const int n_keys = pos0 + rows;
  if (n_keys <= 16) {
    const int n_attn = (n_pairs + 3) / 4;
    const int grid = n_attn + gelu_blocks(gelu);
#define BT_LOCAL_REG(TT, MAXJ) BT_DISPATCH_DH(d_head, (attn_local_reg_kernel<TT, DH, MAXJ><<<grid, 256, 0, s>>>( \
        qkv, (TT*)Kl, (TT*)Vl, rope, (TT*)out, dtype == BT_F32 ? 0 : out_lo_off, n_pairs, n_heads, rot, rows, pos0, l_cap, n_attn, gelu)))
    if (dtype == BT_F32) {
      if (n_keys <= 4) { BT_LOCAL_REG(float, 4); } else if (n_keys <= 8) { BT_LOCAL_REG(float, 8); } else { BT_LOCAL_REG(float, 16); }
    } else {
      if (n_keys <= 4) { BT_LOCAL_REG(bf16_t, 4); } else if (n_keys <= 8) { BT_LOCAL_REG(bf16_t, 8); } else { BT_LOCAL_REG(bf16_t, 16); }
    }
#undef BT_LOCAL_REG
    return hipGetLastError();
  }
  const size_t per_wave = (size_t)(2 * l_cap + 2) * d_head * sizeof(float);
  int nw = 4;
  while (nw > 1 && per_wave * nw > 60 * 1024) nw >>= 1;
  if (per_wave * nw > 60 * 1024) return hipErrorInvalidValue;
  const int n_attn = (n_pairs + nw - 1) / nw;
  const int grid = n_attn + gelu_blocks(gelu);
  const size_t shm = per_wave * nw;
  if (dtype == BT_F32) {
    BT_DISPATCH_DH(d_head, (attn_local_kernel<float, DH><<<grid, nw * 64, shm, s>>>(
        qkv, (float*)Kl, (float*)Vl, rope, (float*)out, 0, n_pairs, n_heads, rot, rows, pos0, l_cap, n_attn, gelu)));
  } else {
    BT_DISPATCH_DH(d_head, (attn_local_kernel<bf16_t, DH><<<grid, nw * 64, shm, s>>>(
        qkv, (bf16_t*)Kl, (bf16_t*)Vl, rope, (bf16_t*)out, out_lo_off, n_pairs, n_heads, rot, rows, pos0, l_cap, n_attn, gelu)));
  }
  return hipGetLastError();
}

}  // namespace bt
