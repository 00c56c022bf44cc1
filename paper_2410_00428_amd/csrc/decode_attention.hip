// Decode attention through a layer's block table (paper Sections 2.1.2 and 2.2: attention of
// one new token over keys/values kept in non-contiguous blocks; Section 3.2.2: the table is the
// layer's own).
//
// The work is HBM-bound: every key and value byte of the context is read once.  A workgroup
// owns one (sequence, kv head, partition of the context); all q heads that share the kv head
// are handled together so the keys/values are fetched once per kv head.  Within a wavefront
// the 16-byte pieces of a 256-byte row sit in adjacent lanes, so a wavefront load covers whole
// rows; a wavefront takes one block (16 tokens, K then V, contiguous in the pool) per step and
// has all of that block's loads in flight before the first use.  Softmax runs online in fp32;
// each group of lanes that shares a token sub-row keeps its own running (max, sum, output) and
// the groups, then the wavefronts, then the partitions are merged with the usual
// exp(m_i - m) weights.
#include "lkv_internal.hpp"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kBlock = 16;  // tokens per KV block these kernels are built for

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kPerPiece = 4;
  __device__ static void unpack(u32x4 w, float *f) {
    f[0] = __uint_as_float(w.x); f[1] = __uint_as_float(w.y); f[2] = __uint_as_float(w.z); f[3] = __uint_as_float(w.w);
  }
  __device__ static void store(float *p, float v) { *p = v; }
};
template <> struct Elem<uint16_t> {  // bfloat16 bit patterns
  static constexpr int kPerPiece = 8;
  __device__ static void unpack(u32x4 w, float *f) {
    f[0] = __uint_as_float(w.x << 16); f[1] = __uint_as_float(w.x & 0xffff0000u);
    f[2] = __uint_as_float(w.y << 16); f[3] = __uint_as_float(w.y & 0xffff0000u);
    f[4] = __uint_as_float(w.z << 16); f[5] = __uint_as_float(w.z & 0xffff0000u);
    f[6] = __uint_as_float(w.w << 16); f[7] = __uint_as_float(w.w & 0xffff0000u);
  }
  __device__ static void store(uint16_t *p, float v) {
    __bf16 b = (__bf16)v;  // round to nearest even
    *p = *reinterpret_cast<uint16_t *>(&b);
  }
};

__device__ __forceinline__ float safe_max(float m) { return m == -INFINITY ? 0.f : m; }

// Partial results of one (sequence, q head, partition): m, l and the unnormalised output row.
struct Workspace {
  float *ml;  // [B][Hq][parts][2]
  float *o;   // [B][Hq][parts][D]
};

template <typename T, int D, int G>
__global__ void __launch_bounds__(kThreads)
paged_decode_kernel(const T *__restrict__ Q, T *__restrict__ O, const char *__restrict__ pool,
                    const int32_t *__restrict__ block_table, int max_blocks, const int32_t *__restrict__ context_lens,
                    int Hq, int64_t block_bytes, float scale, int partition, int num_parts, Workspace ws) {
  constexpr int EPL = Elem<T>::kPerPiece;   // elements per 16-byte piece
  constexpr int LPR = D / EPL;              // lanes per row
  constexpr int TPI = 64 / LPR;             // tokens covered by one wavefront load
  constexpr int NI = kBlock / TPI;          // loads per lane per block, for K and again for V
  constexpr int64_t kRowBytes = (int64_t)D * sizeof(T);

  const int part = blockIdx.x, g = blockIdx.y, s = blockIdx.z;
  const int n = context_lens[s];
  const int start = part * partition;
  if (start >= n && part != 0) return;
  const int end = min(n, start + partition);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane / LPR, c = lane % LPR;

  float q[G][EPL];
#pragma unroll
  for (int j = 0; j < G; ++j) {
    u32x4 w = *(const u32x4 *)(Q + ((int64_t)s * Hq + g * G + j) * D + c * EPL);
    Elem<T>::unpack(w, q[j]);
#pragma unroll
    for (int e = 0; e < EPL; ++e) q[j][e] *= scale;
  }
  float m[G], l[G], acc[G][EPL];
#pragma unroll
  for (int j = 0; j < G; ++j) {
    m[j] = -INFINITY;
    l[j] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[j][e] = 0.f;
  }

  const int32_t *table = block_table + (int64_t)s * max_blocks;
  for (int b = start / kBlock + wave; b * kBlock < end; b += kWaves) {
    const int blk = __builtin_amdgcn_readfirstlane(table[b]);
    const char *base = pool + (int64_t)blk * block_bytes + (int64_t)g * (2 * kBlock * kRowBytes) +
                       (int64_t)r * kRowBytes + c * 16;
    u32x4 kw[NI], vw[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) kw[i] = *(const u32x4 *)(base + (int64_t)i * TPI * kRowBytes);
#pragma unroll
    for (int i = 0; i < NI; ++i) vw[i] = *(const u32x4 *)(base + kBlock * kRowBytes + (int64_t)i * TPI * kRowBytes);

    float sc[G][NI];
    bool valid[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      valid[i] = b * kBlock + i * TPI + r < end;
      float k[EPL];
      Elem<T>::unpack(kw[i], k);
#pragma unroll
      for (int j = 0; j < G; ++j) {
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) d = fmaf(q[j][e], k[e], d);
#pragma unroll
        for (int off = 1; off < LPR; off <<= 1) d += __shfl_xor(d, off);
        sc[j][i] = valid[i] ? d : -INFINITY;  // a masked slot may hold anything, NaN included
      }
    }
#pragma unroll
    for (int j = 0; j < G; ++j) {
      float mn = m[j];
#pragma unroll
      for (int i = 0; i < NI; ++i) mn = fmaxf(mn, sc[j][i]);
      const float ms = safe_max(mn);
      const float alpha = __expf(m[j] - ms);
      m[j] = mn;
      l[j] *= alpha;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[j][e] *= alpha;
#pragma unroll
      for (int i = 0; i < NI; ++i) sc[j][i] = __expf(sc[j][i] - ms);
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      float v[EPL];
      Elem<T>::unpack(vw[i], v);
#pragma unroll
      for (int e = 0; e < EPL; ++e) v[e] = valid[i] ? v[e] : 0.f;
#pragma unroll
      for (int j = 0; j < G; ++j) {
        l[j] += sc[j][i];
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[j][e] = fmaf(sc[j][i], v[e], acc[j][e]);
      }
    }
  }

  // merge the lane groups that worked on different token sub-rows
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const float mo = __shfl_xor(m[j], off), lo = __shfl_xor(l[j], off);
      const float mn = fmaxf(m[j], mo), ms = safe_max(mn);
      const float a = __expf(m[j] - ms), bsc = __expf(mo - ms);
      l[j] = l[j] * a + lo * bsc;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[j][e] = acc[j][e] * a + __shfl_xor(acc[j][e], off) * bsc;
      m[j] = mn;
    }
  }

  // merge the wavefronts through LDS
  __shared__ float sm_ml[kWaves][G][2];
  __shared__ float sm_o[kWaves][G][D];
  if (r == 0) {
#pragma unroll
    for (int j = 0; j < G; ++j) {
      if (c == 0) {
        sm_ml[wave][j][0] = m[j];
        sm_ml[wave][j][1] = l[j];
      }
#pragma unroll
      for (int e = 0; e < EPL; ++e) sm_o[wave][j][c * EPL + e] = acc[j][e];
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < G * D; idx += kThreads) {
    const int j = idx / D, col = idx % D;
    float mn = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) mn = fmaxf(mn, sm_ml[w][j][0]);
    const float ms = safe_max(mn);
    float lt = 0.f, ot = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float a = __expf(sm_ml[w][j][0] - ms);
      lt += sm_ml[w][j][1] * a;
      ot += sm_o[w][j][col] * a;
    }
    const int64_t row = (int64_t)s * Hq + g * G + j;
    if (num_parts == 1) {
      Elem<T>::store(O + row * D + col, lt > 0.f ? ot / lt : 0.f);
    } else {
      const int64_t p = row * num_parts + part;
      ws.o[p * D + col] = ot;
      if (col == 0) {
        ws.ml[p * 2] = mn;
        ws.ml[p * 2 + 1] = lt;
      }
    }
  }
}

// One workgroup per (sequence, q head): merges the partitions that the context spans.
template <typename T, int D>
__global__ void __launch_bounds__(D)
decode_combine_kernel(T *__restrict__ O, const int32_t *__restrict__ context_lens, int Hq, int partition,
                      int num_parts, Workspace ws) {
  const int64_t row = blockIdx.x;
  const int s = (int)(row / Hq), col = threadIdx.x;
  const int n = context_lens[s];
  const int parts = n <= 0 ? 0 : (n + partition - 1) / partition;
  float mn = -INFINITY;
  for (int p = 0; p < parts; ++p) mn = fmaxf(mn, ws.ml[(row * num_parts + p) * 2]);
  const float ms = safe_max(mn);
  float lt = 0.f, ot = 0.f;
  for (int p = 0; p < parts; ++p) {
    const int64_t i = row * num_parts + p;
    const float a = __expf(ws.ml[i * 2] - ms);
    lt += ws.ml[i * 2 + 1] * a;
    ot += ws.o[i * D + col] * a;
  }
  Elem<T>::store(O + row * D + col, lt > 0.f ? ot / lt : 0.f);
}

int pick_partition(const lkv_ctx *c, int num_seqs, int max_blocks) {
  if (c->cfg.decode_partition > 0) return c->cfg.decode_partition;
  const int64_t tokens = (int64_t)max_blocks * kBlock;
  int p = 512;
  while (p > 128 && (int64_t)num_seqs * c->cfg.num_kv_heads * ((tokens + p - 1) / p) < 2048) p >>= 1;
  return p;
}

template <typename T, int D, int G>
hipError_t launch_t(const lkv_ctx *c, const void *Q, void *O, const int32_t *bt, int max_blocks, const int32_t *cl,
                    int num_seqs, float *wsbuf, hipStream_t s) {
  const int partition = pick_partition(c, num_seqs, max_blocks);
  int num_parts = (int)(((int64_t)max_blocks * kBlock + partition - 1) / partition);
  if (num_parts < 1) num_parts = 1;
  const int Hq = c->cfg.num_q_heads;
  Workspace ws{wsbuf, wsbuf + (int64_t)num_seqs * Hq * num_parts * 2};
  hipLaunchKernelGGL((paged_decode_kernel<T, D, G>), dim3(num_parts, c->cfg.num_kv_heads, num_seqs), dim3(kThreads), 0,
                     s, (const T *)Q, (T *)O, c->pool, bt, max_blocks, cl, Hq, c->block_bytes, c->scale, partition,
                     num_parts, ws);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || num_parts == 1) return e;
  hipLaunchKernelGGL((decode_combine_kernel<T, D>), dim3(num_seqs * Hq), dim3(D), 0, s, (T *)O, cl, Hq, partition,
                     num_parts, ws);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_g(const lkv_ctx *c, const void *Q, void *O, const int32_t *bt, int max_blocks, const int32_t *cl,
                    int num_seqs, float *ws, hipStream_t s) {
  switch (c->cfg.num_q_heads / c->cfg.num_kv_heads) {
    case 1: return launch_t<T, D, 1>(c, Q, O, bt, max_blocks, cl, num_seqs, ws, s);
    case 2: return launch_t<T, D, 2>(c, Q, O, bt, max_blocks, cl, num_seqs, ws, s);
    case 4: return launch_t<T, D, 4>(c, Q, O, bt, max_blocks, cl, num_seqs, ws, s);
    case 8: return launch_t<T, D, 8>(c, Q, O, bt, max_blocks, cl, num_seqs, ws, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

namespace lkv {

bool decode_supported(const lkv_ctx *c) {
  const int g = c->cfg.num_q_heads / c->cfg.num_kv_heads;
  return c->cfg.block_size == kBlock && (c->cfg.head_dim == 64 || c->cfg.head_dim == 128) &&
         (g == 1 || g == 2 || g == 4 || g == 8);
}

int64_t decode_workspace_bytes(const lkv_ctx *c, int32_t num_seqs, int32_t max_blocks) {
  const int partition = pick_partition(c, num_seqs, max_blocks);
  const int64_t parts = ((int64_t)max_blocks * kBlock + partition - 1) / partition;
  if (parts <= 1) return 0;
  return (int64_t)num_seqs * c->cfg.num_q_heads * parts * (2 + c->cfg.head_dim) * (int64_t)sizeof(float);
}

hipError_t launch_paged_decode(const lkv_ctx *c, const void *Q, void *O, const int32_t *bt, int32_t max_blocks,
                               const int32_t *cl, int32_t num_seqs, float *ws, hipStream_t s) {
  const bool f32 = c->cfg.dtype == LKV_F32;
  if (c->cfg.head_dim == 64)
    return f32 ? launch_g<float, 64>(c, Q, O, bt, max_blocks, cl, num_seqs, ws, s)
               : launch_g<uint16_t, 64>(c, Q, O, bt, max_blocks, cl, num_seqs, ws, s);
  return f32 ? launch_g<float, 128>(c, Q, O, bt, max_blocks, cl, num_seqs, ws, s)
             : launch_g<uint16_t, 128>(c, Q, O, bt, max_blocks, cl, num_seqs, ws, s);
}

}  // namespace lkv
