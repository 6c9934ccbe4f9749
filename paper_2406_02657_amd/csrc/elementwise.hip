// Embedder gather-concat, token-embedding gather, fused residual + LayerNorm,
// greedy argmax.  All bandwidth-trivial; written for 64-lane wavefronts.
#include "common.h"
#include "kernels.h"
#include "../../include/bt.h"

namespace bt {

// ---------------------------------------------------------------------------
// Embedder (Sec. 2.2): one workgroup per block row; 16-byte chunks of the table
// rows are copied (widened to float) into the residual stream.
// ---------------------------------------------------------------------------
template <class T>
__global__ __launch_bounds__(256) void embed_concat_kernel(const T* __restrict__ E, const int32_t* __restrict__ tokens,
                                                           float* __restrict__ x, int block_len, int d_emb,
                                                           int blocks_per_seq, int row_stride, int seq_len_arg,
                                                           const int* __restrict__ seq_lens, int pad_id) {
  constexpr int EPC = Chunk<T>::EPC;
  const int m = blockIdx.x;
  const int b = m / blocks_per_seq, blk = m - b * blocks_per_seq;
  const int len = seq_lens ? seq_lens[b] : seq_len_arg;
  const int pad = (len + block_len - 1) / block_len * block_len - len;   // pads in front of the sequence's first block
  const int chunks_per_tok = d_emb / EPC;
  const int n_chunks = block_len * chunks_per_tok;
  float* xr = x + (size_t)m * block_len * d_emb;
  for (int c = threadIdx.x; c < n_chunks; c += blockDim.x) {
    const int j = c / chunks_per_tok, cc = c - j * chunks_per_tok;
    const int t = blk * block_len + j - pad;           // index into the unpadded sequence
    // t >= len: a block past the end of a shorter sequence of the batch; its row is never used
    const int tok = (t < 0 || t >= len) ? pad_id : tokens[(size_t)b * row_stride + t];
    const uint4 raw = *reinterpret_cast<const uint4*>(E + (size_t)tok * d_emb + cc * EPC);
    float f[EPC];
    Chunk<T>::unpack(raw, f);
    float* dst = xr + j * d_emb + cc * EPC;
#pragma unroll
    for (int e = 0; e < EPC; e += 4)
      *reinterpret_cast<float4*>(dst + e) = make_float4(f[e], f[e + 1], f[e + 2], f[e + 3]);
  }
}

hipError_t launch_embed_concat(int dtype, const void* E_emb, const int32_t* tokens, float* x,
                               int n_seqs, int blocks_per_seq, int block_len, int d_emb,
                               int row_stride, int seq_len, const int* seq_lens, int pad_id, hipStream_t s) {
  const int n_rows = n_seqs * blocks_per_seq;
  if (n_rows <= 0) return hipSuccess;
  if (!seq_lens && (seq_len < 1 || seq_len > row_stride || seq_len > blocks_per_seq * block_len)) return hipErrorInvalidValue;
  if (dtype == BT_F32)
    embed_concat_kernel<float><<<n_rows, 256, 0, s>>>((const float*)E_emb, tokens, x, block_len, d_emb,
                                                      blocks_per_seq, row_stride, seq_len, seq_lens, pad_id);
  else
    embed_concat_kernel<bf16_t><<<n_rows, 256, 0, s>>>((const bf16_t*)E_emb, tokens, x, block_len, d_emb,
                                                       blocks_per_seq, row_stride, seq_len, seq_lens, pad_id);
  return hipGetLastError();
}

template <class T>
__global__ __launch_bounds__(256) void token_embed_kernel(const T* __restrict__ E, const int32_t* __restrict__ cur,
                                                          float* __restrict__ x, int block_len, int r_prev, int D) {
  constexpr int EPC = Chunk<T>::EPC;
  const int b = blockIdx.x;
  const int tok = cur[b * block_len + r_prev];
  for (int c = threadIdx.x; c < D / EPC; c += blockDim.x) {
    const uint4 raw = *reinterpret_cast<const uint4*>(E + (size_t)tok * D + c * EPC);
    float f[EPC];
    Chunk<T>::unpack(raw, f);
    float* dst = x + (size_t)b * D + c * EPC;
#pragma unroll
    for (int e = 0; e < EPC; e += 4)
      *reinterpret_cast<float4*>(dst + e) = make_float4(f[e], f[e + 1], f[e + 2], f[e + 3]);
  }
}

hipError_t launch_token_embed(int dtype, const void* E_tok, const int32_t* cur, float* x,
                              int batch, int block_len, int r_prev, int d_model, hipStream_t s) {
  if (dtype == BT_F32)
    token_embed_kernel<float><<<batch, 256, 0, s>>>((const float*)E_tok, cur, x, block_len, r_prev, d_model);
  else
    token_embed_kernel<bf16_t><<<batch, 256, 0, s>>>((const bf16_t*)E_tok, cur, x, block_len, r_prev, d_model);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Residual update + LayerNorm.  One workgroup (256 threads) per row; a thread
// owns VPT groups of four consecutive floats, kept in registers (D <= 1024*VPT).
// The split-K partial sums of the two producing GEMMs are added in a fixed order
// (deterministic); all loads of a thread are issued together, without branches.
// Mean and biased variance are taken in two passes over the registers, as the
// definition states them.
// ---------------------------------------------------------------------------
constexpr int kLnThreads = 256;

__device__ __forceinline__ float block_sum_256(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

__device__ __forceinline__ void add4(float4& a, const float4& b) { a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w; }

// acc += sum over the splits of partA, then of partB, of the float4 at element offset off.
// The two lists are walked as one, kLnBatch loads in flight at a time and no branch around
// them: indices past the end are clamped (the value is then multiplied by zero).
constexpr int kLnBatch = 24;
template <int BATCH>
__device__ __forceinline__ void add_partials(float4& acc, const float* partA, int nA, const float* partB, int nB,
                                             size_t stride, size_t off) {
  const int n = nA + nB;
  for (int s0 = 0; s0 < n; s0 += BATCH) {
    float4 v[BATCH];
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      const int s = min(s0 + u, n - 1);
      const float* p = s < nA ? partA + (size_t)s * stride : partB + (size_t)(s - nA) * stride;
      v[u] = *reinterpret_cast<const float4*>(p + off);
    }
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      const float k = (s0 + u < n) ? 1.f : 0.f;
      acc.x += k * v[u].x; acc.y += k * v[u].y; acc.z += k * v[u].z; acc.w += k * v[u].w;
    }
  }
}

// What the kernel receives.  Every workgroup fetches its kernel arguments from memory before it can
// issue anything else, and each further 64-byte line of them lengthens that first trip, so the
// fields every launch needs fit two lines (LnHot) and the rarely used ones (LnCold) are a second
// argument that only the EXTRA instantiation touches.
struct LnHot {
  float* x;
  const float *partA, *partB, *biasA, *biasB;
  const float *g1, *b1, *g2, *b2;
  void *u1, *u2;
  size_t part_stride;
  unsigned lo_off;
  int D, in_mul, in_off;
  float eps;
  unsigned packed;       // splitsA | splitsB << 12 | u1_f32 << 24 | write_x << 25
};
static_assert(sizeof(LnHot) <= 128, "two cache lines");
struct LnCold {
  const void* emb_table;
  const int32_t* emb_ids;
  int* counter_inc;
  const int* in_off_dev;
  const float* add;          // summation token decoder: row i also gets add[i * add_stride + col]
  int emb_stride, emb_off, add_stride;
};

template <class T, int VPT, bool EXTRA, int BATCH = kLnBatch>
__device__ __forceinline__ void resid_ln_body(const LnHot& a, const LnCold& cold) {
  __shared__ float red[4];
  const int i = blockIdx.x;
  const int in_off = (EXTRA && cold.in_off_dev) ? cold.in_off_dev[i] - 1 : a.in_off;
  const size_t row = (size_t)i * a.in_mul + in_off;
  const int D = a.D, G = D >> 2;
  const int splitsA = a.packed & 0xfff, splitsB = (a.packed >> 12) & 0xfff;
  const bool u1_f32 = (a.packed >> 24) & 1, write_x = (a.packed >> 25) & 1;
  const void* emb_table = EXTRA ? cold.emb_table : nullptr;
  int* counter_inc = EXTRA ? cold.counter_inc : nullptr;
  constexpr bool kEarly = VPT == 1;           // one group per thread: gamma / beta ride along the first trip to memory
  float4 v[VPT], g1e, b1e, g2e, b2e;
  float* xr = a.x + row * D;
  const int nA = a.partA ? splitsA : 0, nB = a.partB ? splitsB : 0;
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
  // Every load of the kernel is issued here, before the first reduction: one trip to memory.
#pragma unroll
  for (int c = 0; c < VPT; ++c) {
    const int g = min((int)threadIdx.x + c * kLnThreads, G - 1);     // clamped: no branch around the loads
    if constexpr (kEarly) {
      g1e = *reinterpret_cast<const float4*>(a.g1 + 4 * g);
      b1e = *reinterpret_cast<const float4*>(a.b1 + 4 * g);
      g2e = a.g2 ? *reinterpret_cast<const float4*>(a.g2 + 4 * g) : zero;
      b2e = a.g2 ? *reinterpret_cast<const float4*>(a.b2 + 4 * g) : zero;
    }
    float4 acc;
    const float* add = EXTRA ? cold.add : nullptr;
    if (emb_table) {
      const T* er = reinterpret_cast<const T*>(emb_table) + (size_t)cold.emb_ids[(size_t)i * cold.emb_stride + cold.emb_off] * D + 4 * g;
      acc = make_float4(to_float<T>(er[0]), to_float<T>(er[1]), to_float<T>(er[2]), to_float<T>(er[3]));
    } else if (add) {
      acc = zero;                                   // the row is the added vector alone
    } else {
      acc = *reinterpret_cast<const float4*>(xr + 4 * g);
    }
    if (add) add4(acc, *reinterpret_cast<const float4*>(add + (size_t)i * cold.add_stride + 4 * g));
    if (nA && a.biasA) add4(acc, *reinterpret_cast<const float4*>(a.biasA + 4 * g));
    if (nB && a.biasB) add4(acc, *reinterpret_cast<const float4*>(a.biasB + 4 * g));
    if (nA + nB) add_partials<BATCH>(acc, a.partA, nA, a.partB, nB, a.part_stride, row * D + 4 * g);
    v[c] = acc;
  }
  if (counter_inc && threadIdx.x == 0) counter_inc[i] += 1;
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < VPT; ++c) {
    const bool live = (int)threadIdx.x + c * kLnThreads < G;
    if (live) {
      if (write_x) *reinterpret_cast<float4*>(xr + 4 * (threadIdx.x + c * kLnThreads)) = v[c];
      sum += (v[c].x + v[c].y) + (v[c].z + v[c].w);
    }
  }
  const float mean = block_sum_256(sum, red) / (float)D;
  float sq = 0.f;
#pragma unroll
  for (int c = 0; c < VPT; ++c) {
    if ((int)threadIdx.x + c * kLnThreads < G) {
      const float t0 = v[c].x - mean, t1 = v[c].y - mean, t2 = v[c].z - mean, t3 = v[c].w - mean;
      sq += (t0 * t0 + t1 * t1) + (t2 * t2 + t3 * t3);
    }
  }
  const float var = block_sum_256(sq, red) / (float)D;
  const float rstd = 1.0f / sqrtf(var + a.eps);
#pragma unroll
  for (int c = 0; c < VPT; ++c) {
    const int g = threadIdx.x + c * kLnThreads;
    if (g < G) {
      const float n[4] = {(v[c].x - mean) * rstd, (v[c].y - mean) * rstd, (v[c].z - mean) * rstd, (v[c].w - mean) * rstd};
      float4 g1, b1;
      if constexpr (kEarly) { g1 = g1e; b1 = b1e; }
      else { g1 = *reinterpret_cast<const float4*>(a.g1 + 4 * g); b1 = *reinterpret_cast<const float4*>(a.b1 + 4 * g); }
      const float o1[4] = {n[0] * g1.x + b1.x, n[1] * g1.y + b1.y, n[2] * g1.z + b1.z, n[3] * g1.w + b1.w};
      const size_t o = (size_t)i * D + 4 * g;
      if (u1_f32) {
        *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.u1) + o) = make_float4(o1[0], o1[1], o1[2], o1[3]);
      } else {
        store_act4<T>(reinterpret_cast<T*>(a.u1), o, a.lo_off, o1[0], o1[1], o1[2], o1[3]);
      }
      if (a.g2) {
        float4 g2, b2;
        if constexpr (kEarly) { g2 = g2e; b2 = b2e; }
        else { g2 = *reinterpret_cast<const float4*>(a.g2 + 4 * g); b2 = *reinterpret_cast<const float4*>(a.b2 + 4 * g); }
        const float o2[4] = {n[0] * g2.x + b2.x, n[1] * g2.y + b2.y, n[2] * g2.z + b2.z, n[3] * g2.w + b2.w};
        store_act4<T>(reinterpret_cast<T*>(a.u2), o, a.lo_off, o2[0], o2[1], o2[2], o2[3]);
      }
    }
  }
}

template <class T, int VPT>
__global__ __launch_bounds__(kLnThreads) __attribute__((amdgpu_waves_per_eu(1, 2))) void resid_ln_kernel(LnHot a) {
  resid_ln_body<T, VPT, false>(a, LnCold{});
}
// With the rarely used inputs: rows gathered from an embedding table, the per-sequence block
// counters, per-row offsets from device memory.
template <class T, int VPT>
__global__ __launch_bounds__(kLnThreads) __attribute__((amdgpu_waves_per_eu(1, 2))) void resid_ln_extra_kernel(LnHot a, LnCold c) {
  resid_ln_body<T, VPT, true>(a, c);
}

// Many rows (prefill, scoring, large batches): the same body without the occupancy cap and with
// the partial sums taken four at a time (such launches have two pieces, not twenty).  The cap and
// the deep batch buy the 64-row decode launches registers for their loads; with thousands of rows
// it is resident workgroups, not registers, that keep enough bytes in flight.
template <class T, int VPT>
__global__ __launch_bounds__(kLnThreads) void resid_ln_many_kernel(LnHot a) {
  resid_ln_body<T, VPT, false, 4>(a, LnCold{});
}

template <class T>
static hipError_t launch_resid_ln_t(const ResidLnArgs& r, hipStream_t s, const int* in_off_dev) {
  const int G = r.D / 4;
  if (G > 4 * kLnThreads) return hipErrorInvalidValue;
  if (r.splitsA < 0 || r.splitsA > 0xfff || r.splitsB < 0 || r.splitsB > 0xfff || r.lo_off > 0xffffffffu) return hipErrorInvalidValue;
  LnHot a;
  a.x = r.x; a.partA = r.partA; a.partB = r.partB; a.biasA = r.biasA; a.biasB = r.biasB;
  a.g1 = r.g1; a.b1 = r.b1; a.g2 = r.g2; a.b2 = r.b2; a.u1 = r.u1; a.u2 = r.u2;
  a.part_stride = r.part_stride; a.lo_off = (unsigned)r.lo_off; a.D = r.D; a.in_mul = r.in_mul; a.in_off = r.in_off;
  a.eps = r.eps;
  a.packed = (unsigned)r.splitsA | (unsigned)r.splitsB << 12 | (r.u1_f32 ? 1u << 24 : 0u) | (r.write_x ? 1u << 25 : 0u);
  if (r.emb_table || r.counter_inc || in_off_dev || r.add) {
    const LnCold c{r.emb_table, r.emb_ids, r.counter_inc, in_off_dev, r.add, r.emb_stride, r.emb_off, r.add_stride};
    if (G <= kLnThreads) resid_ln_extra_kernel<T, 1><<<r.n_rows, kLnThreads, 0, s>>>(a, c);
    else if (G <= 2 * kLnThreads) resid_ln_extra_kernel<T, 2><<<r.n_rows, kLnThreads, 0, s>>>(a, c);
    else resid_ln_extra_kernel<T, 4><<<r.n_rows, kLnThreads, 0, s>>>(a, c);
  } else if (r.n_rows >= 1024) {
    if (G <= kLnThreads) resid_ln_many_kernel<T, 1><<<r.n_rows, kLnThreads, 0, s>>>(a);
    else if (G <= 2 * kLnThreads) resid_ln_many_kernel<T, 2><<<r.n_rows, kLnThreads, 0, s>>>(a);
    else resid_ln_many_kernel<T, 4><<<r.n_rows, kLnThreads, 0, s>>>(a);
  } else {
    if (G <= kLnThreads) resid_ln_kernel<T, 1><<<r.n_rows, kLnThreads, 0, s>>>(a);
    else if (G <= 2 * kLnThreads) resid_ln_kernel<T, 2><<<r.n_rows, kLnThreads, 0, s>>>(a);
    else resid_ln_kernel<T, 4><<<r.n_rows, kLnThreads, 0, s>>>(a);
  }
  return hipGetLastError();
}

hipError_t launch_resid_ln(int dtype, const ResidLnArgs& a, hipStream_t s, const int* in_off_dev) {
  if (a.n_rows <= 0) return hipSuccess;
  if (a.D % 4) return hipErrorInvalidValue;
  return dtype == BT_F32 ? launch_resid_ln_t<float>(a, s, in_off_dev) : launch_resid_ln_t<bf16_t>(a, s, in_off_dev);
}

// ---------------------------------------------------------------------------
// Greedy argmax, lowest index on ties.  One workgroup of 1024 threads per
// sequence; each thread scans 16-byte groups of logits (all loads independent),
// then wave shuffles and one pass over the 16 wave results.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void argmax_take(float v, int i, float& best, int& bi) {
  if (v > best || (v == best && i < bi)) { best = v; bi = i; }
}

// End-of-sequence rule (eos_id >= 0): a sequence that has emitted eos_id emits eos_id from then on.
__device__ __forceinline__ int apply_eos(int id, int eos_id, int32_t* finished, int b) {
  if (eos_id < 0) return id;
  if (finished[b]) return eos_id;
  if (id == eos_id) finished[b] = 1;
  return id;
}

__device__ __forceinline__ void argmax_body(const float* __restrict__ logits, int vocab,
                                            int32_t* __restrict__ next_ids, int32_t* __restrict__ cur,
                                            int block_len, int r, int eos_id, int32_t* __restrict__ finished) {
  __shared__ float sv[16];
  __shared__ int si[16];
  const int b = blockIdx.x;
  const float* lg = logits + (size_t)b * vocab;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  if ((vocab & 3) == 0) {
    const float4* lg4 = reinterpret_cast<const float4*>(lg);
    for (int g = threadIdx.x; g < vocab / 4; g += 1024) {
      const float4 q = lg4[g];
      argmax_take(q.x, 4 * g, best, bi);
      argmax_take(q.y, 4 * g + 1, best, bi);
      argmax_take(q.z, 4 * g + 2, best, bi);
      argmax_take(q.w, 4 * g + 3, best, bi);
    }
  } else {
    for (int v = threadIdx.x; v < vocab; v += 1024) argmax_take(lg[v], v, best, bi);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(best, o, kWave);
    const int oi = __shfl_xor(bi, o, kWave);
    argmax_take(ov, oi, best, bi);
  }
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = best; si[threadIdx.x >> 6] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 16; ++w) argmax_take(sv[w], si[w], best, bi);
    if (bi == 0x7fffffff) bi = 0;           // every logit was NaN or -inf
    bi = apply_eos(bi, eos_id, finished, b);
    if (next_ids) next_ids[b] = bi;
    cur[b * block_len + r] = bi;
  }
}

// Two entry points each: the one without the end-of-sequence rule keeps the short argument list.
__global__ __launch_bounds__(1024) void argmax_kernel(const float* __restrict__ logits, int vocab,
                                                      int32_t* __restrict__ next_ids, int32_t* __restrict__ cur,
                                                      int block_len, int r) {
  argmax_body(logits, vocab, next_ids, cur, block_len, r, -1, nullptr);
}
__global__ __launch_bounds__(1024) void argmax_eos_kernel(const float* __restrict__ logits, int vocab,
                                                          int32_t* __restrict__ next_ids, int32_t* __restrict__ cur,
                                                          int block_len, int r, int eos_id, int32_t* __restrict__ finished) {
  argmax_body(logits, vocab, next_ids, cur, block_len, r, eos_id, finished);
}

hipError_t launch_argmax(const float* logits, int batch, int vocab, int32_t* next_ids,
                         int32_t* cur, int block_len, int r, int eos_id, int32_t* finished, hipStream_t s) {
  if (eos_id >= 0) argmax_eos_kernel<<<batch, 1024, 0, s>>>(logits, vocab, next_ids, cur, block_len, r, eos_id, finished);
  else argmax_kernel<<<batch, 1024, 0, s>>>(logits, vocab, next_ids, cur, block_len, r);
  return hipGetLastError();
}

// Greedy argmax from per-tile candidates: one wave per sequence scans cand[b * n_tiles + tile].
__device__ __forceinline__ void argmax_candidates_body(const float2* __restrict__ cand, int n_tiles, int vocab,
                                                       int32_t* __restrict__ next_ids, int32_t* __restrict__ cur,
                                                       int block_len, int r, int eos_id, int32_t* __restrict__ finished) {
  const int b = blockIdx.x;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int t = threadIdx.x; t < n_tiles; t += 64) {
    const float2 c = cand[(size_t)b * n_tiles + t];
    argmax_take(c.x, __float_as_int(c.y), best, bi);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(best, o, kWave);
    const int oi = __shfl_xor(bi, o, kWave);
    argmax_take(ov, oi, best, bi);
  }
  if (threadIdx.x == 0) {
    // every logit was NaN or -inf; or the column is not one: the id indexes the embedding table in the
    // next step, so a candidate buffer its producer did not fill must not turn into a wild row
    if ((unsigned)bi >= (unsigned)vocab) bi = 0;
    bi = apply_eos(bi, eos_id, finished, b);
    if (next_ids) next_ids[b] = bi;
    cur[b * block_len + r] = bi;
  }
}

__global__ __launch_bounds__(64) void argmax_candidates_kernel(const float2* __restrict__ cand, int n_tiles, int vocab,
                                                               int32_t* __restrict__ next_ids, int32_t* __restrict__ cur,
                                                               int block_len, int r) {
  argmax_candidates_body(cand, n_tiles, vocab, next_ids, cur, block_len, r, -1, nullptr);
}
__global__ __launch_bounds__(64) void argmax_candidates_eos_kernel(const float2* __restrict__ cand, int n_tiles, int vocab,
                                                                   int32_t* __restrict__ next_ids, int32_t* __restrict__ cur,
                                                                   int block_len, int r, int eos_id,
                                                                   int32_t* __restrict__ finished) {
  argmax_candidates_body(cand, n_tiles, vocab, next_ids, cur, block_len, r, eos_id, finished);
}

hipError_t launch_argmax_candidates(const float2* cand, int n_tiles, int batch, int vocab, int32_t* next_ids,
                                    int32_t* cur, int block_len, int r, int eos_id, int32_t* finished, hipStream_t s) {
  if (n_tiles < 1 || vocab < 1) return hipErrorInvalidValue;
  if (eos_id >= 0) argmax_candidates_eos_kernel<<<batch, 64, 0, s>>>(cand, n_tiles, vocab, next_ids, cur, block_len, r, eos_id, finished);
  else argmax_candidates_kernel<<<batch, 64, 0, s>>>(cand, n_tiles, vocab, next_ids, cur, block_len, r);
  return hipGetLastError();
}

__global__ void scatter_ids_kernel(const int32_t* __restrict__ ids, int32_t* __restrict__ cur, int batch,
                                   int block_len, int r, int eos_id, int32_t* __restrict__ finished) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < batch) {
    cur[b * block_len + r] = ids[b];
    if (eos_id >= 0 && ids[b] == eos_id) finished[b] = 1;     // a forced end-of-sequence id ends the sequence too
  }
}

hipError_t launch_scatter_ids(const int32_t* ids, int32_t* cur, int batch, int block_len, int r, int eos_id,
                              int32_t* finished, hipStream_t s) {
  if (batch <= 0) return hipErrorInvalidValue;
  scatter_ids_kernel<<<(batch + 255) / 256, 256, 0, s>>>(ids, cur, batch, block_len, r, eos_id, finished);
  return hipGetLastError();
}

// dst[i] = src[i] for n 16-byte chunks (a kernel rather than a copy node, so that the launch may sit
// in a captured graph next to the others).
__global__ void copy16_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

hipError_t launch_copy16(void* dst, const void* src, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  if ((bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return hipErrorInvalidValue;
  const size_t n = bytes / 16;
  copy16_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(reinterpret_cast<uint4*>(dst), reinterpret_cast<const uint4*>(src), n);
  return hipGetLastError();
}

__global__ void gather_ids_kernel(const int32_t* __restrict__ cur, int32_t* __restrict__ out, int batch,
                                  int block_len, int r) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < batch) out[b] = cur[b * block_len + r];
}

hipError_t launch_gather_ids(const int32_t* cur, int32_t* out, int batch, int block_len, int r, hipStream_t s) {
  gather_ids_kernel<<<(batch + 255) / 256, 256, 0, s>>>(cur, out, batch, block_len, r);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Teacher-forced scoring (Sec. 2.1, all blocks in parallel).  Local sequence s = bl * (N - 1) + j
// scores block j + 1 of sequence bl of the chunk from the context embedding of block j; it has
// Lq = P + L_B - 1 rows: the P prefix rows, then the block's first L_B - 1 token embeddings.
// ---------------------------------------------------------------------------
template <class T>
__global__ __launch_bounds__(256) void score_assemble_kernel(const float* __restrict__ pref, const T* __restrict__ E_tok,
                                                             const int32_t* __restrict__ tokens, float* __restrict__ x,
                                                             int D, int P, int block_len, int n_blocks, int seq_len) {
  const int Lq = P + block_len - 1;
  const int pad = n_blocks * block_len - seq_len;      // the first block was completed from the left
  const int row = blockIdx.x;
  const int s = row / Lq, pos = row - s * Lq;
  const int bl = s / (n_blocks - 1), j = s - bl * (n_blocks - 1);
  float* dst = x + (size_t)row * D;
  if (pos < P) {
    const float* src = pref + ((size_t)(bl * n_blocks + j) * P + pos) * D;
    for (int i = threadIdx.x * 4; i < D; i += 1024) *reinterpret_cast<float4*>(dst + i) = *reinterpret_cast<const float4*>(src + i);
  } else {
    const int tok = tokens[(size_t)bl * seq_len + (j + 1) * block_len + (pos - P) - pad];
    const T* src = E_tok + (size_t)tok * D;
    for (int i = threadIdx.x * 4; i < D; i += 1024)
      *reinterpret_cast<float4*>(dst + i) = make_float4(to_float<T>(src[i]), to_float<T>(src[i + 1]), to_float<T>(src[i + 2]), to_float<T>(src[i + 3]));
  }
}

hipError_t launch_score_assemble(int dtype, const float* pref, const void* E_tok, const int32_t* tokens, float* x,
                                 int n_seqs, int n_blocks, int seq_len, int D, int P, int block_len, hipStream_t s) {
  const int rows = n_seqs * (n_blocks - 1) * (P + block_len - 1);
  if (rows <= 0) return hipSuccess;
  if (D % 4 || P < 1 || n_blocks < 2) return hipErrorInvalidValue;
  if (dtype == BT_F32)
    score_assemble_kernel<float><<<rows, 256, 0, s>>>(pref, (const float*)E_tok, tokens, x, D, P, block_len, n_blocks, seq_len);
  else
    score_assemble_kernel<bf16_t><<<rows, 256, 0, s>>>(pref, (const bf16_t*)E_tok, tokens, x, D, P, block_len, n_blocks, seq_len);
  return hipGetLastError();
}

// One workgroup per logits row: nll = log(sum exp(z - max)) + max - z[target].  Rows at the first
// P - 1 prefix positions predict nothing and are skipped.
__global__ __launch_bounds__(1024) void score_rows_kernel(const float* __restrict__ logits, int vocab, int row0,
                                                          const int32_t* __restrict__ tokens, float* __restrict__ nll,
                                                          int P, int block_len, int n_blocks, int seq_len) {
  __shared__ float red[16];
  const int Lq = P + block_len - 1;
  const int row = row0 + blockIdx.x;
  const int s = row / Lq, pos = row - s * Lq;
  if (pos < P - 1) return;
  const int bl = s / (n_blocks - 1), j = s - bl * (n_blocks - 1);
  const size_t t = (size_t)bl * seq_len + (j + 1) * block_len + (pos - (P - 1)) - (n_blocks * block_len - seq_len);
  const float* z = logits + (size_t)blockIdx.x * vocab;
  float mx = -INFINITY;
  for (int v = threadIdx.x; v < vocab; v += 1024) mx = fmaxf(mx, z[v]);
  mx = wave_max(mx);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
  __syncthreads();
  mx = red[0];
#pragma unroll
  for (int w = 1; w < 16; ++w) mx = fmaxf(mx, red[w]);
  __syncthreads();
  float sum = 0.f;
  for (int v = threadIdx.x; v < vocab; v += 1024) sum += expf(z[v] - mx);
  sum = wave_sum(sum);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sum;
  __syncthreads();
  if (threadIdx.x == 0) {
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) tot += red[w];
    nll[t] = logf(tot) + mx - z[tokens[t]];
  }
}

// Target column per token-decoder row of a chunk (row = s * Lq + pos as above): the token the row
// predicts, or -1 for the first P - 1 prefix positions.
__global__ void score_targets_kernel(const int32_t* __restrict__ tokens, int32_t* __restrict__ targets, int n_rows,
                                     int P, int block_len, int n_blocks, int seq_len) {
  const int row = blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= n_rows) return;
  const int Lq = P + block_len - 1;
  const int s = row / Lq, pos = row - s * Lq;
  const int bl = s / (n_blocks - 1), j = s - bl * (n_blocks - 1);
  targets[row] = pos < P - 1 ? -1 : tokens[(size_t)bl * seq_len + (j + 1) * block_len + (pos - (P - 1)) - (n_blocks * block_len - seq_len)];
}

hipError_t launch_score_targets(const int32_t* tokens, int32_t* targets, int n_rows, int P, int block_len,
                                int n_blocks, int seq_len, hipStream_t s) {
  if (n_rows <= 0) return hipSuccess;
  score_targets_kernel<<<(n_rows + 255) / 256, 256, 0, s>>>(tokens, targets, n_rows, P, block_len, n_blocks, seq_len);
  return hipGetLastError();
}

// nll from the pieces a GEMM with the log-sum-exp epilogue left: one wave per row combines the
// (max, sum of exponentials) of its column groups.
__global__ __launch_bounds__(256) void score_combine_kernel(const float2* __restrict__ stats, int groups,
                                                            const float* __restrict__ target_logit, int n_rows, int row0,
                                                            float* __restrict__ nll, int P, int block_len, int n_blocks,
                                                            int seq_len) {
  const int lane = threadIdx.x & 63;
  const int local = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (local >= n_rows) return;
  const int Lq = P + block_len - 1;
  const int row = row0 + local;
  const int s = row / Lq, pos = row - s * Lq;
  if (pos < P - 1) return;
  const int bl = s / (n_blocks - 1), j = s - bl * (n_blocks - 1);
  const size_t t = (size_t)bl * seq_len + (j + 1) * block_len + (pos - (P - 1)) - (n_blocks * block_len - seq_len);
  const float2* st = stats + (size_t)local * groups;
  float m = -INFINITY;
  for (int g = lane; g < groups; g += 64) m = fmaxf(m, st[g].x);
  m = wave_max(m);
  float sum = 0.f;
  for (int g = lane; g < groups; g += 64) {
    const float2 p = st[g];
    sum += p.y > 0.f ? p.y * __expf(p.x - m) : 0.f;
  }
  sum = wave_sum(sum);
  if (lane == 0) nll[t] = logf(sum) + m - target_logit[local];
}

hipError_t launch_score_combine(const float2* stats, int groups, const float* target_logit, int n_rows, int row0,
                                float* nll, int P, int block_len, int n_blocks, int seq_len, hipStream_t s) {
  if (n_rows <= 0) return hipSuccess;
  score_combine_kernel<<<(n_rows + 3) / 4, 256, 0, s>>>(stats, groups, target_logit, n_rows, row0, nll, P, block_len,
                                                         n_blocks, seq_len);
  return hipGetLastError();
}

hipError_t launch_score_rows(const float* logits, int n_rows, int vocab, int row0, const int32_t* tokens, float* nll,
                             int P, int block_len, int n_blocks, int seq_len, hipStream_t s) {
  if (n_rows <= 0) return hipSuccess;
  score_rows_kernel<<<n_rows, 1024, 0, s>>>(logits, vocab, row0, tokens, nll, P, block_len, n_blocks, seq_len);
  return hipGetLastError();
}

// Rotary table: tab[pos * (rot/2) + t] = (cos, sin) of pos * 10000^(-2t/rot), evaluated in double.
__global__ void rope_table_kernel(float2* __restrict__ tab, int n_pos, int rot) {
  const int half = rot / 2;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)n_pos * half) return;
  const int pos = (int)(i / half), t = (int)(i - (size_t)pos * half);
  const double ang = (double)pos * pow(10000.0, -2.0 * (double)t / (double)rot);
  tab[i] = make_float2((float)cos(ang), (float)sin(ang));
}

hipError_t launch_rope_table(float2* tab, int n_pos, int rot, hipStream_t s) {
  if (n_pos <= 0 || rot < 2 || (rot & 1)) return hipErrorInvalidValue;
  const size_t n = (size_t)n_pos * (rot / 2);
  rope_table_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(tab, n_pos, rot);
  return hipGetLastError();
}

__global__ void state_set_kernel(int* p, int value, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = value;
}
__global__ void seq_blocks_kernel(const int* lens, int* n_blocks, int block_len, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) n_blocks[i] = (lens[i] + block_len - 1) / block_len;
}

hipError_t launch_state_set(int* p, int value, int n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  state_set_kernel<<<(n + 255) / 256, 256, 0, s>>>(p, value, n);
  return hipGetLastError();
}
hipError_t launch_seq_blocks(const int* lens, int* n_blocks, int block_len, int n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  seq_blocks_kernel<<<(n + 255) / 256, 256, 0, s>>>(lens, n_blocks, block_len, n);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Calibration probes: what a plain kernel reaches on this chip, to set beside the published peaks.
// ---------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(4))) unsigned probe_u32x4_t;
__global__ __launch_bounds__(256) void probe_read_kernel(const probe_u32x4_t* __restrict__ src, size_t chunks_per_wg, float* __restrict__ out) {
  const probe_u32x4_t* p = src + (size_t)blockIdx.x * chunks_per_wg + threadIdx.x;
  probe_u32x4_t acc = {0u, 0u, 0u, 0u};
  // a workgroup walks its own contiguous range, 4 KB per step, eight independent loads in flight per thread
  size_t c = 0;
  for (; c + 8 * 256 <= chunks_per_wg; c += 8 * 256) {
    probe_u32x4_t v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(p + c + u * 256);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
  }
  for (; c < chunks_per_wg; c += 256) acc ^= __builtin_nontemporal_load(p + c);
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = __uint_as_float((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) & 0x3fffffffu);
}

hipError_t launch_probe_read(const void* src, size_t bytes, int workgroups, float* out, hipStream_t s) {
  if (!src || !out || workgroups <= 0 || bytes == 0 || bytes % ((size_t)workgroups * 256 * 16)) return hipErrorInvalidValue;
  probe_read_kernel<<<workgroups, 256, 0, s>>>(reinterpret_cast<const probe_u32x4_t*>(src), bytes / 16 / workgroups, out);
  return hipGetLastError();
}

typedef __attribute__((ext_vector_type(4))) float probe_f32x4_t;
typedef __attribute__((ext_vector_type(8))) __bf16 probe_bf16x8_t;
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, int random_operands, float* __restrict__ out) {
  probe_f32x4_t acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = probe_f32x4_t{0.f, 0.f, 0.f, 0.f};
  probe_bf16x8_t a, b;
  unsigned x = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    x = x * 1664525u + 1013904223u;
    const float ra = ((int)((x >> 8) % 2001u) - 1000) * 1e-3f;
    x = x * 1664525u + 1013904223u;
    const float rb = ((int)((x >> 8) % 2001u) - 1000) * 1e-3f;
    a[i] = (__bf16)(random_operands ? ra : (float)(threadIdx.x & 3));
    b[i] = (__bf16)(random_operands ? rb : 1.0f);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) sum += (acc[i][0] + acc[i][1]) + (acc[i][2] + acc[i][3]);
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = sum;
}

hipError_t launch_probe_mfma(int iters, int random_operands, int workgroups, float* out, hipStream_t s) {
  if (!out || iters <= 0 || workgroups <= 0) return hipErrorInvalidValue;
  probe_mfma_kernel<<<workgroups, 256, 0, s>>>(iters, random_operands, out);
  return hipGetLastError();
}

}  // namespace bt
