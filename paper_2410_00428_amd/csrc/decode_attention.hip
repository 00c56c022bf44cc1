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
#include <mutex>
#include <type_traits>

// Split-K partial results for callers that cannot allocate device memory (lkv_paged_decode_attention_static): a fixed
// array in the library's device image, one copy per GPU at that GPU's own address.  In host code the name `scratch`
// is only a handle for hipGetSymbolAddress; the kernels get the address that call returns, like any other buffer.
static __device__ __align__(256) unsigned char scratch[LKV_STATIC_DECODE_SCRATCH_BYTES];

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// A context never reaches past its row of the block table: a longer one (a caller's mistake) is cut there, so that
// no table entry outside the row is read and no partition outside the grid is expected.
__device__ __forceinline__ int capped(int n, int cap) { return n < cap ? n : cap; }
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

// Sum over the LPR adjacent lanes that hold one row; every lane of the group gets the total.
// Steps inside a 16-lane row are DPP adds (no LDS traffic); only a 32-lane row needs a shuffle.
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, false));
}
template <int LPR>
__device__ __forceinline__ float row_sum(float x) {
  if (LPR >= 2) x += dpp_mov<0xB1>(x);                       // quad_perm [1,0,3,2]
  if (LPR >= 4) x += dpp_mov<0x4E>(x);                       // quad_perm [2,3,0,1]
  if (LPR == 8) x += dpp_mov<0x141>(x);                      // row_half_mirror: the other quad of the 8
  if (LPR >= 16) { x += dpp_mov<0x124>(x); x += dpp_mov<0x128>(x); }  // row_ror 4, row_ror 8
  if (LPR >= 32) x += __shfl_xor(x, 16);
  return x;
}

template <typename T> __device__ __forceinline__ float fexp(float x);
template <> __device__ __forceinline__ float fexp<float>(float x) { return expf(x); }       // fp32 parity path
template <> __device__ __forceinline__ float fexp<uint16_t>(float x) { return __expf(x); }

template <typename T, int D, int G, int WAVES>
__global__ void __launch_bounds__(WAVES * 64)
paged_decode_kernel(const T *__restrict__ Q, T *__restrict__ O, const char *__restrict__ pool,
                    const int32_t *__restrict__ block_table, int max_blocks, const int32_t *__restrict__ context_lens,
                    int Hq, int group, int64_t block_bytes, int pool_blocks, float scale, int partition, int num_parts,
                    Workspace ws) {
  // G is the register capacity: the kernel serves `group` <= G query heads per kv head (the heads past `group`
  // repeat the last one and are dropped at the end), so that 3, 5, 6 and 7 heads per kv head run as 4 resp. 8.
  constexpr int EPL = Elem<T>::kPerPiece;   // elements per 16-byte piece
  constexpr int LPR = D / EPL;              // lanes per row
  constexpr int TPI = 64 / LPR;             // tokens covered by one wavefront load
  constexpr int NI = kBlock / TPI;          // loads per lane per block, for K and again for V
  constexpr int64_t kRowBytes = (int64_t)D * sizeof(T);
  constexpr bool kPrefetch = G <= 2;        // two blocks in flight per wavefront while registers allow

  const int g = blockIdx.x, s = blockIdx.y, part = blockIdx.z;  // partition index slowest: see make_plan
  const int n = capped(context_lens[s], max_blocks * kBlock);
  const int start = part * partition;
  if (start >= n && part != 0) return;
  const int end = min(n, start + partition);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane / LPR, c = lane % LPR;

  float q[G][EPL];
#pragma unroll
  for (int j = 0; j < G; ++j) {
    u32x4 w = *(const u32x4 *)(Q + ((int64_t)s * Hq + g * group + min(j, group - 1)) * D + c * EPL);
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

  // This wavefront's blocks: first, first+WAVES, ...  Their table entries are fetched 64 at a time,
  // one per lane, and broadcast from that register as the loop reaches them.
  const int first = start / kBlock + wave, nb_end = (end + kBlock - 1) / kBlock;
  const int iters = first < nb_end ? (nb_end - first + WAVES - 1) / WAVES : 0;
  const int32_t *table = block_table + (int64_t)s * max_blocks;
  const char *lane_base = pool + (int64_t)g * (2 * kBlock * kRowBytes) + (int64_t)r * kRowBytes + c * 16;

  for (int it0 = 0; it0 < iters; it0 += 64) {
    const int cnt = min(64, iters - it0);
    // an entry outside the pool is a caller error (e.g. a context longer than the table): clamp it so that
    // the result is wrong but nothing outside the pool is read
    const int my_entry = lane < cnt ? min(max(table[first + (it0 + lane) * WAVES], 0), pool_blocks - 1) : 0;

    auto load = [&](int it, u32x4 *kw, u32x4 *vw) {
      const int blk = __builtin_amdgcn_readlane(my_entry, it);
      const char *base = lane_base + (int64_t)blk * block_bytes;
#pragma unroll
      for (int i = 0; i < NI; ++i) kw[i] = __builtin_nontemporal_load((const u32x4 *)(base + (int64_t)i * TPI * kRowBytes));
#pragma unroll
      for (int i = 0; i < NI; ++i)
        vw[i] = __builtin_nontemporal_load((const u32x4 *)(base + kBlock * kRowBytes + (int64_t)i * TPI * kRowBytes));
    };
    auto compute = [&](int it, const u32x4 *kw, const u32x4 *vw) {
      const int tok0 = (first + (it0 + it) * WAVES) * kBlock + r;
      float sc[G][NI];
      bool valid[NI];
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        valid[i] = tok0 + i * TPI < end;
        float k[EPL];
        Elem<T>::unpack(kw[i], k);
#pragma unroll
        for (int j = 0; j < G; ++j) {
          float d = 0.f;
#pragma unroll
          for (int e = 0; e < EPL; ++e) d = fmaf(q[j][e], k[e], d);
          d = row_sum<LPR>(d);
          sc[j][i] = valid[i] ? d : -INFINITY;  // a masked slot may hold anything, NaN included
        }
      }
#pragma unroll
      for (int j = 0; j < G; ++j) {
        float mn = m[j];
#pragma unroll
        for (int i = 0; i < NI; ++i) mn = fmaxf(mn, sc[j][i]);
        const float ms = safe_max(mn);
        const float alpha = fexp<T>(m[j] - ms);
        m[j] = mn;
        l[j] *= alpha;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[j][e] *= alpha;
#pragma unroll
        for (int i = 0; i < NI; ++i) sc[j][i] = fexp<T>(sc[j][i] - ms);
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
    };

    if (kPrefetch) {
      u32x4 ka[NI], va[NI], kb[NI], vb[NI];
      load(0, ka, va);
      for (int it = 0; it < cnt; it += 2) {
        if (it + 1 < cnt) load(it + 1, kb, vb);
        compute(it, ka, va);
        if (it + 1 < cnt) {
          if (it + 2 < cnt) load(it + 2, ka, va);
          compute(it + 1, kb, vb);
        }
      }
    } else {
      u32x4 ka[NI], va[NI];
      for (int it = 0; it < cnt; ++it) {
        load(it, ka, va);
        compute(it, ka, va);
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
      const float a = fexp<T>(m[j] - ms), bsc = fexp<T>(mo - ms);
      l[j] = l[j] * a + lo * bsc;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[j][e] = acc[j][e] * a + __shfl_xor(acc[j][e], off) * bsc;
      m[j] = mn;
    }
  }

  // merge the wavefronts through LDS
  __shared__ float sm_ml[WAVES][G][2];
  __shared__ float sm_o[WAVES][G][D];
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
  for (int idx = threadIdx.x; idx < group * D; idx += WAVES * 64) {
    const int j = idx / D, col = idx % D;
    float mn = -INFINITY;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) mn = fmaxf(mn, sm_ml[w][j][0]);
    const float ms = safe_max(mn);
    float lt = 0.f, ot = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const float a = fexp<T>(sm_ml[w][j][0] - ms);
      lt += sm_ml[w][j][1] * a;
      ot += sm_o[w][j][col] * a;
    }
    const int64_t row = (int64_t)s * Hq + g * group + j;
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

// ------------------------------------------------------------------------------------------
// bf16, head_dim 128, any group size up to 16: the same streaming scheme with both products on the
// matrix cores (v_mfma_f32_16x16x32_bf16), so that grouped-query heads cost no extra vector work.
// A wavefront takes a PAIR of blocks (32 keys) per step.  Lane l = (c = l%16, hq = l/16).
//   S^T = K Q^T   A operand: lane (c, hq) holds 16 bytes of key row kappa(c), taken straight from the
//                 pool; two MFMA chains X and Y cover the pair with kappa_X(c) = 8*(c/4) + c%4 and
//                 kappa_Y = kappa_X + 4, so that afterwards lane (q = c, hq) holds the scores of keys
//                 8*hq .. 8*hq+7 of the pair: exactly the B operand of the second product.
//   O^T = V^T P^T A operand: lane (c, hq) loads the 16-byte piece c of value rows 8*hq .. 8*hq+7
//                 (a 16-lane group reads whole 256-byte rows) and transposes the 8x8 bf16 patch in
//                 registers with v_perm_b32; patch row i is the operand of MFMA i, whose 16 output
//                 rows are the channels 8*c + i.  Lane (q, hq) ends up with channels 32*hq .. 32*hq+31.
// Rows of masked keys are zeroed before the product (a masked slot may hold NaN).
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 v = __builtin_convertvector(f, bf16x2);  // round to nearest even
  return __builtin_bit_cast(unsigned, v);
}

// Which (sequence, partition) a workgroup of the one-dimensional grid works on.  The host sizes the grid from
// the table width (it cannot see the context lengths), so every workgroup derives the launch's work list from
// context_lens itself: rank 0.. are the FULL partitions of all sequences in sequence order, then come the
// partial last partitions (and the empty contexts, whose partition 0 writes the zero row), longest first.  The
// hardware starts workgroups in rank order and a CU takes a new one when it is done with the last, so the work
// that is left for the end of the launch is the smallest: a ragged batch does not end on a few CUs streaming a
// whole partition each while the rest of the chip is idle.  Ranks past the list have nothing to do.
// Every lane returns the same (seq, part); seq < 0 = nothing to do.  Built for num_seqs <= 256.
__device__ __forceinline__ void decode_work_item(const int32_t *__restrict__ context_lens, int num_seqs, int partition,
                                                 int cap, int rank, int &seq, int &part) {
  const int lane = threadIdx.x & 63;
  if (num_seqs <= 64) {
    // the whole batch fits one register per lane: one load, scalar walks over the lanes (v_readlane)
    const int n = lane < num_seqs ? capped(context_lens[lane], cap) : -1;
    const int f = n > 0 ? n / partition : 0;                                          // full partitions
    const int r = n == 0 ? 0 : (n > 0 && n % partition != 0) ? n % partition : -1;   // remainder, -1 = none
    int acc = 0;
    seq = -1;
    part = 0;
    for (int k = 0; k < num_seqs; ++k) {
      const int fk = __builtin_amdgcn_readlane(f, k);
      if (rank >= acc && rank < acc + fk) {
        seq = k;
        part = rank - acc;
      }
      acc += fk;
    }
    if (seq >= 0) return;
    const int r_rank = rank - acc;
    if (r_rank >= __popcll(__ballot(r >= 0))) return;  // past the end of the work list
    int my_rank = 0;
    for (int k = 0; k < num_seqs; ++k) {
      const int rk = __builtin_amdgcn_readlane(r, k);
      if (rk > r || (rk == r && k < lane)) ++my_rank;
    }
    const unsigned long long win = __ballot(r >= 0 && my_rank == r_rank);
    const int w = __ffsll((long long)win) - 1;  // exactly one lane
    seq = w;
    part = __builtin_amdgcn_readlane(f, w);
    return;
  }
  int found = -1, found_part = 0, base_rank = 0;
  // full partitions, sequence order
  for (int b0 = 0; b0 < num_seqs; b0 += 64) {
    const int s = b0 + lane;
    const int n = s < num_seqs ? capped(context_lens[s], cap) : 0;
    const int f = n > 0 ? n / partition : 0;
    int incl = f;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int up = __shfl_up(incl, d);
      if (lane >= d) incl += up;
    }
    const int excl = base_rank + incl - f;
    if (rank >= excl && rank < excl + f) {
      found = s;
      found_part = rank - excl;
    }
    base_rank += __shfl(incl, 63);
  }
  unsigned long long hit = __ballot(found >= 0);
  if (hit) {
    const int src = __ffsll((long long)hit) - 1;
    seq = __shfl(found, src);
    part = __shfl(found_part, src);
    return;
  }
  // partial partitions: the rank-th largest remainder (ties: lower sequence index first).  The search is
  // quadratic in the batch size; the host uses this order for batches of at most 256 sequences.
  const int r_rank = rank - base_rank;
  int num_cand = 0;
  for (int b0 = 0; b0 < num_seqs; b0 += 64) {
    const int s = b0 + lane;
    const int n = s < num_seqs ? capped(context_lens[s], cap) : -1;
    num_cand += __popcll(__ballot(n == 0 || (n > 0 && n % partition != 0)));
  }
  if (r_rank >= num_cand) {  // past the end of the work list
    seq = -1;
    part = 0;
    return;
  }
  for (int b0 = 0; b0 < num_seqs; b0 += 64) {
    const int s = b0 + lane;
    const int n = s < num_seqs ? capped(context_lens[s], cap) : -1;
    const bool cand = n == 0 || (n > 0 && n % partition != 0);
    const int r = n > 0 ? n % partition : 0;
    int my_rank = 0;
    for (int t0 = 0; t0 < num_seqs; t0 += 64) {
      const int t = t0 + lane;
      const int nt = t < num_seqs ? capped(context_lens[t], cap) : -1;
      // remainder of sequence t, or -1 if it has no partial partition (never counted: r >= 0)
      const int rt = nt == 0 ? 0 : (nt > 0 && nt % partition != 0) ? nt % partition : -1;
      const int kmax = min(64, num_seqs - t0);
      for (int k = 0; k < kmax; ++k) {  // k is uniform: the broadcast is a v_readlane, not an LDS shuffle
        const int rk = __builtin_amdgcn_readlane(rt, k);
        if (rk > r || (rk == r && t0 + k < s)) ++my_rank;
      }
    }
    if (cand && my_rank == r_rank) {
      found = s;
      found_part = n > 0 ? n / partition : 0;
    }
  }
  hit = __ballot(found >= 0);
  if (hit) {
    const int src = __ffsll((long long)hit) - 1;
    seq = __shfl(found, src);
    part = __shfl(found_part, src);
  } else {
    seq = -1;
    part = 0;
  }
}

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
// Eight E4M3 codes -> eight bf16 values (exact: every E4M3 value is a bf16 value); two codes per instruction.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x4 widen_e4m3(u32x2 w) {
  return u32x4{__builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w.x, 1.0f, false)),
               __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w.x, 1.0f, true)),
               __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w.y, 1.0f, false)),
               __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w.y, 1.0f, true))};
}

// What a lane loads per access: 16 bytes = 8 bf16 channels, or 8 bytes = 8 E4M3 codes.
// The lane's 8 key channels of product step kk as bf16: bf16 keys are loaded one step per load, 8-bit keys two.
template <bool FP8> __device__ __forceinline__ u32x4 key_piece(const u32x4 *k, int kk) {
  if constexpr (FP8) {
    const u32x4 w = k[kk >> 1];
    return (kk & 1) ? widen_e4m3(u32x2{w.z, w.w}) : widen_e4m3(u32x2{w.x, w.y});
  } else {
    return k[kk];
  }
}
// Channels 2T, 2T+1 of a lane's 8 channels as one word of two bf16.
template <int T> __device__ __forceinline__ unsigned bf16_pair(u32x4 w) { return w[T]; }
template <int T> __device__ __forceinline__ unsigned bf16_pair(u32x2 w) {
  return __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[T >> 1], 1.0f, (T & 1) != 0));
}

// How the workgroups of a launch find their work.
enum DecodeOrder {
  kOrderPlain = 0,    // workgroup rank -> (sequence, partition), sequence fastest
  kOrderLongest = 1,  // the launch's (sequence, partition) items longest first (decode_work_item)
  kOrderEven = 2      // every workgroup takes the same number of key pairs, whatever sequences they belong to
};
constexpr int kMaxEvenSeqs = 256;  // batch size up to which the even split is built
// Even split: what one (sequence, kv head) row costs on the line of work, in units of one key pair: its pairs plus
// kRowCost for starting and finishing a piece (first table entries and keys behind dependent loads, the merge of the
// wavefronts: a few microseconds, against ~0.7 us of streaming per pair at a CU's share of the HBM rate; 8 measured
// best among 4, 8 and 12).
constexpr int kRowCost = 8;
__device__ __forceinline__ int even_row_cost(int tokens) {
  return tokens > 0 ? (tokens + 2 * kBlock - 1) / (2 * kBlock) + kRowCost : 0;
}

template <int G, int WAVES, bool FP8>
__global__ void __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(2)))  // two wavefronts per SIMD
paged_decode_mfma_kernel(const uint16_t *__restrict__ Q, uint16_t *__restrict__ O, const char *__restrict__ pool,
                         const int32_t *__restrict__ block_table, int max_blocks,
                         const int32_t *__restrict__ context_lens, int Hq, int group, int64_t block_bytes,
                         int pool_blocks, float scale, float out_scale, int partition, int num_parts, int num_seqs,
                         int order, Workspace ws) {
  // G is the capacity (LDS rows of the merge) for `group` <= G query heads per kv head: the heads are columns of
  // the matrix products, of which there are 16 whatever the group size.
  // FP8: the pool holds one-byte E4M3 codes (rows of 128 bytes, pieces of 8 channels = 8 bytes); they are widened
  // to bf16 in registers (exact) and take the same path; the K scale is part of `scale`, the V scale is out_scale.
  constexpr int D = 128;
  constexpr int kRow = FP8 ? D : D * 2;  // bytes per key/value row
  constexpr int kPiece = FP8 ? 8 : 16;   // bytes of 8 channels
  constexpr int kDepth = 2;              // block pairs in flight per wavefront
  constexpr int kKeyLoads = FP8 ? 2 : 4; // 16-byte loads per key row and lane
  using Piece = std::conditional_t<FP8, u32x2, u32x4>;
  __shared__ float sm_ml[WAVES][G][2];
  __shared__ float sm_o[WAVES][G][D];
  const int Hkv = Hq / group;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, hq = lane >> 4;

  // One piece of work: keys [start, end) of sequence s (n cached tokens) for kv head g.  The result goes to O when
  // ws_base < 0 (the piece is the whole context), else the partial (m, l, o) of query head j of the group goes to
  // entry ws_base + j * ws_stride of the workspace.
  auto piece = [&](const int s, const int g, const int start, const int end, const int64_t ws_base,
                   const int64_t ws_stride) {
  bf16x8 qop[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    u32x4 w = {0, 0, 0, 0};
    // which 8 channels the lane holds in product step kk: any split of the 128 channels over (kk, hq) will do as
    // long as keys and queries use the same one; the 8-bit layout lets a lane take 16 codes of a key with one load
    const int ch = FP8 ? 64 * (kk >> 1) + 16 * hq + 8 * (kk & 1) : 32 * kk + 8 * hq;
    if (c < group) w = *(const u32x4 *)(Q + ((int64_t)s * Hq + g * group + c) * D + ch);
    qop[kk] = __builtin_bit_cast(bf16x8, w);
  }
  f32x4 oacc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) oacc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m = -INFINITY, l = 0.f;

  const int nb_begin = start / kBlock, nb_end = (end + kBlock - 1) / kBlock;
  const int npairs = (nb_end - nb_begin + 1) / 2;
  const int my_pairs = wave < npairs ? (npairs - wave + WAVES - 1) / WAVES : 0;
  const int32_t *table = block_table + (int64_t)s * max_blocks;
  // byte offsets inside a (block, head) run for the two roles of this lane
  const int k_off = (8 * ((c >> 2) & 1) + (c & 3)) * kRow + 16 * hq;       // key row kappa_X(c) % 16, 16 bytes at hq
  const int v_off = kBlock * kRow + 8 * (hq & 1) * kRow + kPiece * c;       // value rows 8*(hq%2)..+7, piece c
  const bool k_second = c >= 8, v_second = hq >= 2;                     // which block of the pair
  const int64_t head_off = (int64_t)g * (2 * kBlock * kRow);

  for (int p0 = 0; p0 < my_pairs; p0 += 32) {
    const int cnt = min(32, my_pairs - p0);
    // lane i keeps the table entry of block i%2 of this wavefront's (p0 + i/2)-th pair
    const int bidx = nb_begin + 2 * (wave + (p0 + (lane >> 1)) * WAVES) + (lane & 1);
    // an entry outside the pool is a caller error (e.g. a context longer than the table): clamp it so that
    // the result is wrong but nothing outside the pool is read; -1 marks "no second block" in a pair
    const int my_entry = (lane < 2 * cnt && bidx < nb_end) ? min(max(table[bidx], 0), pool_blocks - 1) : -1;

    // K and V are read exactly once per launch: non-temporal loads keep them from displacing each other in L2 and
    // the last-level cache on their way through (measured: 6.0 -> 6.45 TB/s on 64 long contexts, 5.5 -> 5.9 TB/s
    // on 8 x 2049 tokens)
    auto load = [&](int it, u32x4 *kx, u32x4 *ky, Piece *vr) {
      const int id0 = __builtin_amdgcn_readlane(my_entry, 2 * it);
      int id1 = __builtin_amdgcn_readlane(my_entry, 2 * it + 1);
      if (id1 < 0) id1 = id0;  // odd block count: the pair's second half is fully masked
      const char *b0 = pool + (int64_t)id0 * block_bytes + head_off;
      const char *b1 = pool + (int64_t)id1 * block_bytes + head_off;
      const char *kb = (k_second ? b1 : b0) + k_off;
      const char *vb = (v_second ? b1 : b0) + v_off;
#pragma unroll
      for (int j = 0; j < kKeyLoads; ++j) kx[j] = __builtin_nontemporal_load((const u32x4 *)(kb + 64 * j));
#pragma unroll
      for (int j = 0; j < kKeyLoads; ++j) ky[j] = __builtin_nontemporal_load((const u32x4 *)(kb + 4 * kRow + 64 * j));
#pragma unroll
      for (int j = 0; j < 8; ++j) vr[j] = __builtin_nontemporal_load((const Piece *)(vb + j * kRow));
    };
    auto compute = [&](int it, const u32x4 *kx, const u32x4 *ky, Piece *vr) {
      const int key0 = (nb_begin + 2 * (wave + (p0 + it) * WAVES)) * kBlock + 8 * hq;  // this lane's 8 keys
      f32x4 sx = {0.f, 0.f, 0.f, 0.f}, sy = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {  // 8-bit codes are widened piece by piece, right before their product
        sx = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, key_piece<FP8>(kx, kk)), qop[kk], sx, 0, 0, 0);
        sy = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, key_piece<FP8>(ky, kk)), qop[kk], sy, 0, 0, 0);
      }
      float t[8];
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        t[v] = key0 + v < end ? sx[v] * scale : -INFINITY;
        t[4 + v] = key0 + 4 + v < end ? sy[v] * scale : -INFINITY;
      }
      float mx = t[0];
#pragma unroll
      for (int e = 1; e < 8; ++e) mx = fmaxf(mx, t[e]);
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float mn = fmaxf(m, mx), ms = safe_max(mn);
      const float alpha = __expf(m - ms);
      m = mn;
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        t[e] = __expf(t[e] - ms);
        psum += t[e];
      }
      l = l * alpha + psum;
#pragma unroll
      for (int i = 0; i < 8; ++i) oacc[i] *= alpha;
      u32x4 pw = {pack_bf16(t[0], t[1]), pack_bf16(t[2], t[3]), pack_bf16(t[4], t[5]), pack_bf16(t[6], t[7])};
      const bf16x8 pb = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (key0 + j >= end) vr[j] = Piece{};  // a masked slot may hold anything (the zero code is 0.0)
      // 8x8 transpose of 16-bit elements: channel pair t of key rows 2w, 2w+1 -> word w of patch rows 2t, 2t+1
      auto channel_pair = [&](auto tc) {
        constexpr int T = decltype(tc)::value;
        unsigned word[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) word[j] = bf16_pair<T>(vr[j]);
#pragma unroll
        for (int i = 2 * T; i < 2 * T + 2; ++i) {
          const unsigned sel = (i & 1) ? 0x07060302u : 0x05040100u;
          u32x4 a;
#pragma unroll
          for (int w = 0; w < 4; ++w) a[w] = __builtin_amdgcn_perm(word[2 * w + 1], word[2 * w], sel);
          oacc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), pb, oacc[i], 0, 0, 0);
        }
      };
      channel_pair(std::integral_constant<int, 0>{});
      channel_pair(std::integral_constant<int, 1>{});
      channel_pair(std::integral_constant<int, 2>{});
      channel_pair(std::integral_constant<int, 3>{});
    };

    // kDepth block pairs in flight per wavefront: the loads of pair it + kDepth - 1 are issued before the math of
    // pair it.  Measured: three pairs of bf16 do not fit the registers (spills, 40 % slower); three or four pairs of
    // 8-bit codes fit and change nothing (what bounds the 8-bit kernel is the number of load instructions: taking a
    // key's codes 16 bytes at a time instead of 8 gave 8-12 %).
    u32x4 kxb[kDepth][kKeyLoads], kyb[kDepth][kKeyLoads];
    Piece vb[kDepth][8];
#pragma unroll
    for (int d = 0; d < kDepth - 1; ++d)
      if (d < cnt) load(d, kxb[d], kyb[d], vb[d]);
    for (int it = 0; it < cnt; it += kDepth) {
#pragma unroll
      for (int d = 0; d < kDepth; ++d) {
        if (it + d < cnt) {
          constexpr int kAhead = kDepth - 1;
          if (it + d + kAhead < cnt) load(it + d + kAhead, kxb[(d + kAhead) % kDepth], kyb[(d + kAhead) % kDepth], vb[(d + kAhead) % kDepth]);
          compute(it + d, kxb[d], kyb[d], vb[d]);
        }
      }
    }
  }
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);

  // merge the wavefronts through LDS; lane (q, hq) owns channels 32*hq + 8*v + i of query q
  if (c < group) {
    if (hq == 0) {
      sm_ml[wave][c][0] = m;
      sm_ml[wave][c][1] = l;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int v = 0; v < 4; ++v) sm_o[wave][c][32 * hq + 8 * v + i] = oacc[i][v];
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < group * D; idx += WAVES * 64) {
    const int j = idx / D, col = idx % D;
    float mn = -INFINITY;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) mn = fmaxf(mn, sm_ml[w][j][0]);
    const float ms = safe_max(mn);
    float lt = 0.f, ot = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const float a = __expf(sm_ml[w][j][0] - ms);
      lt += sm_ml[w][j][1] * a;
      ot += sm_o[w][j][col] * a;
    }
    if (ws_base < 0) {
      const int64_t row = (int64_t)s * Hq + g * group + j;
      Elem<uint16_t>::store(O + row * D + col, lt > 0.f ? ot / lt * out_scale : 0.f);
    } else {
      const int64_t p = ws_base + j * ws_stride;
      ws.o[p * D + col] = ot;
      if (col == 0) {
        ws.ml[p * 2] = mn;
        ws.ml[p * 2 + 1] = lt;
      }
    }
  }
  };  // piece

  if (order == kOrderEven) {
    // Even split.  The (sequence, kv head) rows of the launch, sequence-major, form one line on which a row takes its
    // key pairs (32 keys each) plus kRowCost units in front of them (what starting and finishing a piece costs a
    // workgroup, in pairs' worth of streaming); workgroup w takes the units [w * C, (w + 1) * C) of the line,
    // C = ceil(total / workgroups): every workgroup gets the same amount of work, whatever the mix of context
    // lengths, and a row cut by a workgroup boundary gets one partial result per workgroup that holds some of its
    // pairs.  Partial (row r, workgroup w) lives in workspace entry r + w: along the line either r or w or both
    // grow from one piece to the next, so the entries are distinct, rows + workgroups in all.
    __shared__ int sm_cost[kMaxEvenSeqs], sm_before[kMaxEvenSeqs + 1], sm_tokens[kMaxEvenSeqs];
    for (int i = threadIdx.x; i < num_seqs; i += WAVES * 64) {
      const int t = capped(context_lens[i], max_blocks * kBlock);
      sm_tokens[i] = t;
      sm_cost[i] = even_row_cost(t);
    }
    __syncthreads();
    if (wave == 0) {  // running sum of the sequences' costs, 64 sequences at a time
      int carry = 0;
      for (int i0 = 0; i0 < num_seqs; i0 += 64) {
        const int v = i0 + lane < num_seqs ? sm_cost[i0 + lane] : 0;
        int incl = v;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
          const int up = __shfl_up(incl, d);
          if (lane >= d) incl += up;
        }
        if (i0 + lane < num_seqs) sm_before[i0 + lane] = carry + incl - v;
        carry += __shfl(incl, 63);
      }
      if (lane == 0) sm_before[num_seqs] = carry;
    }
    __syncthreads();
    const int total = Hkv * sm_before[num_seqs];
    const int per_wg = (total + (int)gridDim.x - 1) / (int)gridDim.x;
    int x = (int)blockIdx.x * per_wg;
    const int x_end = min(x + per_wg, total);
    if (x >= x_end) return;
    int lo = 0, hi = num_seqs;  // the last sequence whose first unit is not behind x (it is not empty: x < total)
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (Hkv * sm_before[mid] <= x) lo = mid; else hi = mid;
    }
    int s = lo;
    while (x < x_end) {
      const int cost = sm_cost[s], off = x - Hkv * sm_before[s];
      const int g = off / cost, at = off - g * cost;
      const int take = min(cost - at, x_end - x);
      const int first = max(at - kRowCost, 0), last = max(at + take - kRowCost, 0);  // the pairs among these units
      if (last > first) {
        piece(s, g, first * 2 * kBlock, min(sm_tokens[s], last * 2 * kBlock), ((int64_t)s * Hkv + g + blockIdx.x) * group, 1);
        __syncthreads();  // the merge buffers are used again by the next piece
      }
      x += take;
      if (at + take == cost && g == Hkv - 1) {
        do ++s; while (s < num_seqs && sm_cost[s] == 0);
      }
    }
    return;
  }
  const int g = blockIdx.x % Hkv;  // kv head fastest: workgroups go round-robin to the XCDs
  int s = blockIdx.x / Hkv, part = 0;  // no context is split: one item per sequence
  if (num_parts > 1) {
    if (order == kOrderLongest) {
      decode_work_item(context_lens, num_seqs, partition, max_blocks * kBlock, blockIdx.x / Hkv, s, part);
    } else {
      const int rank = blockIdx.x / Hkv;
      s = rank % num_seqs;
      part = rank / num_seqs;
      if (part * partition >= capped(context_lens[s], max_blocks * kBlock) && part != 0) s = -1;
    }
  }
  if (s < 0) return;
  const int n = capped(context_lens[s], max_blocks * kBlock);
  const int start = part * partition;
  piece(s, g, start, min(n, start + partition), num_parts == 1 ? -1 : ((int64_t)s * Hq + g * group) * num_parts + part,
        num_parts);
}

// The merge of an evenly split launch (kOrderEven): one workgroup per (sequence, q head) finds the workgroups of the
// first kernel that touched its row, from the same running sums, and merges their partial results.
template <typename T, int D>
__global__ void __launch_bounds__(D)
decode_combine_even_kernel(T *__restrict__ O, const int32_t *__restrict__ context_lens, int cap, int Hq, int group,
                           int num_seqs, int num_wgs, float out_scale, Workspace ws) {
  constexpr int kWaves = D / 64;
  const int s = blockIdx.x / Hq, h = blockIdx.x % Hq, col = threadIdx.x;
  const int Hkv = Hq / group, g = h / group, j = h % group;
  __shared__ int sm_int[3][kWaves];
  __shared__ float sm_red[2][kWaves];
  __shared__ float sm_weight[1024];  // per piece: exp(m_w - m); the host launches at most this many workgroups
  int before = 0, all = 0, mine = 0;
  for (int i = threadIdx.x; i < num_seqs; i += D) {
    const int cost = even_row_cost(capped(context_lens[i], cap));
    all += cost;
    if (i < s) before += cost;
    if (i == s) mine = cost;
  }
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) {
    before += __shfl_xor(before, d);
    all += __shfl_xor(all, d);
    mine += __shfl_xor(mine, d);
  }
  if ((threadIdx.x & 63) == 0) {
    sm_int[0][threadIdx.x >> 6] = before;
    sm_int[1][threadIdx.x >> 6] = all;
    sm_int[2][threadIdx.x >> 6] = mine;
  }
  __syncthreads();
  before = all = mine = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    before += sm_int[0][w];
    all += sm_int[1][w];
    mine += sm_int[2][w];
  }
  float lt = 0.f, ot = 0.f;
  if (mine > 0) {  // uniform over the workgroup
    const int total = Hkv * all, per_wg = (total + num_wgs - 1) / num_wgs;
    const int x0 = Hkv * before + g * mine + kRowCost;             // the row's first pair on the line
    const int w_first = x0 / per_wg, pieces = (x0 + mine - kRowCost - 1) / per_wg - w_first + 1;
    const int64_t base = ((int64_t)s * Hkv + g + w_first) * group + j;
    // the pieces' maxima and sums side by side (one piece per thread and round), then their weights
    float mn = -INFINITY;
    for (int w = threadIdx.x; w < pieces; w += D) mn = fmaxf(mn, ws.ml[(base + (int64_t)w * group) * 2]);
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) mn = fmaxf(mn, __shfl_xor(mn, d));
    if ((threadIdx.x & 63) == 0) sm_red[0][threadIdx.x >> 6] = mn;
    __syncthreads();
    mn = sm_red[0][0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) mn = fmaxf(mn, sm_red[0][w]);
    const float ms = safe_max(mn);
    for (int w = threadIdx.x; w < pieces; w += D) {
      const int64_t i = base + (int64_t)w * group;
      const float a = fexp<T>(ws.ml[i * 2] - ms);
      sm_weight[w] = a;
      lt += ws.ml[i * 2 + 1] * a;
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) lt += __shfl_xor(lt, d);
    if ((threadIdx.x & 63) == 0) sm_red[1][threadIdx.x >> 6] = lt;
    __syncthreads();
    lt = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) lt += sm_red[1][w];
#pragma unroll 8
    for (int w = 0; w < pieces; ++w) ot += ws.o[(base + (int64_t)w * group) * D + col] * sm_weight[w];
  }
  Elem<T>::store(O + (int64_t)blockIdx.x * D + col, lt > 0.f ? ot / lt * out_scale : 0.f);
}

// One workgroup per (sequence, q head): merges the partitions that the context spans.
template <typename T, int D>
__global__ void __launch_bounds__(D)
decode_combine_kernel(T *__restrict__ O, const int32_t *__restrict__ context_lens, int cap, int Hq, int partition,
                      int num_parts, float out_scale, Workspace ws) {
  const int64_t row = blockIdx.x;
  const int s = (int)(row / Hq), col = threadIdx.x;
  const int n = capped(context_lens[s], cap);
  const int parts = n <= 0 ? 0 : (n + partition - 1) / partition;
  float mn = -INFINITY;
  for (int p = 0; p < parts; ++p) mn = fmaxf(mn, ws.ml[(row * num_parts + p) * 2]);
  const float ms = safe_max(mn);
  float lt = 0.f, ot = 0.f;
  for (int p = 0; p < parts; ++p) {
    const int64_t i = row * num_parts + p;
    const float a = fexp<T>(ws.ml[i * 2] - ms);
    lt += ws.ml[i * 2 + 1] * a;
    ot += ws.o[i * D + col] * a;
  }
  Elem<T>::store(O + row * D + col, lt > 0.f ? ot / lt * out_scale : 0.f);
}

// Tunables of the split: tokens per partition and wavefronts per workgroup.  The host cannot see
// the context lengths (they live in device memory), so it sizes the grid from the table width.
// The partition index is the SLOWEST grid dimension: workgroups are dealt round-robin to the 8 XCDs,
// and with the partition fastest a short last partition (e.g. 2049 = 2048 + 1 tokens) would put all
// the heavy workgroups on half of the XCDs.
struct Plan {
  int partition, num_parts, waves;
  bool mfma;
  bool lpt;  // workgroups take the launch's (sequence, partition) items longest first (see decode_work_item)
  // even split (kOrderEven): even_wgs workgroups share the launch's key pairs equally; 0 = not used
  int even_wgs;
};

Plan make_plan(const lkv_ctx *c, int num_seqs, int max_blocks) {
  const int64_t tokens = (int64_t)max_blocks * kBlock;
  const int64_t units = (int64_t)num_seqs * c->cfg.num_kv_heads;
  Plan p{0, 1, 4, false, false, 0};
  p.mfma = (c->cfg.dtype == LKV_BF16 || c->cfg.dtype == LKV_FP8_E4M3) && c->cfg.head_dim == 128;
  if (p.mfma) {
    // Measured on MI355X (sweep of partition 256..4096 x 2/4/8 wavefronts over batches of 1..256 sequences, contexts
    // of 200..16384 tokens, MHA and 8-fold GQA): partitions of 4096 tokens when the batch alone fills the chip
    // (contexts up to 4096 are then not split at all), halved until the launch has at least 128 workgroups (one
    // 16384-token GQA sequence: 52 -> 28 us; one 2048-token MHA sequence: 26 -> 15 us).
    p.partition = 4096;
    while (p.partition > 256 && units * ((tokens + p.partition - 1) / p.partition) < 128) p.partition >>= 1;
  } else {
    p.partition = 512;
    while (p.partition > 128 && units * ((tokens + p.partition - 1) / p.partition) < 2048) p.partition >>= 1;
  }
  if (c->cfg.decode_partition > 0) p.partition = c->cfg.decode_partition;
  p.num_parts = (int)((tokens + p.partition - 1) / p.partition);
  if (p.num_parts < 1) p.num_parts = 1;
  // eight wavefronts share a workgroup's keys, except for many short items: with 512 or more workgroups of at most
  // 1024 tokens each, two-wavefront workgroups (four resident per CU) lose less to start-up and the wave merge
  // (256 contexts of 200 tokens: 218 -> 162 us; long items stream better with eight: ragged 16-sequence GQA batch
  // 5.2 vs 4.3 TB/s)
  if (p.mfma) p.waves = (units * p.num_parts >= 512 && (tokens < p.partition ? tokens : p.partition) <= 1024) ? 2 : 8;
  // Longest-first order pays when the launch is only a few rounds of workgroups deep: measured on a ragged
  // 16-sequence GQA batch +26%; with thousands of workgroups the tail is short anyway and the per-workgroup
  // search of the work list costs 2-4%.
  static int cus = 0;
  if (cus == 0 && hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device) != hipSuccess) cus = 256;
  p.lpt = p.mfma && num_seqs <= 256 && units * p.num_parts <= (int64_t)8 * cus;
  // A split launch is cut evenly instead of into partitions of a fixed size: one workgroup per CU, every one with the
  // same share of the launch's key pairs (kOrderEven), whatever the contexts' lengths.  A partitioned launch ends
  // when the CU with the largest items ends, pays the start-up and the merge once per partition, and needs small
  // partitions to give every CU something when the rows (sequences x kv heads) are few.  Measured on MI355X,
  // partitioned -> even: one 16384-token context of the 70B shape 31 -> 26 us, four 8192-token contexts of it
  // 42 -> 35 us; ragged batches (contexts uniform in 128..16384) of the 70B shape with 16 / 64 / 128 / 256 sequences
  // 87.8 -> 84.1 / 452 -> 408 / 752 -> 658 / 1490 -> 1359 us, of the 7B shape with 4 / 16 / 32 / 64 sequences
  // 85 -> 80 / 282 -> 274 / 822 -> 796 / 1519 -> 1479 us; 4 x 16385 tokens x 32 heads 180 either way; the worst
  // case seen is 3 % behind (48 ragged sequences of the 7B shape).  A partition size set by the caller keeps the
  // partitioned launch, and so do batches of more than kMaxEvenSeqs sequences.
  if (p.mfma && p.num_parts > 1 && c->cfg.decode_partition == 0 && num_seqs <= kMaxEvenSeqs &&
      units * (tokens / (2 * kBlock) + 1 + kRowCost) < ((int64_t)1 << 30)) {
    p.even_wgs = cus < 1024 ? cus : 1024;  // the merge kernel keeps one weight per workgroup in LDS
    p.waves = 8;
  }
  return p;
}

template <typename T, int D, int G, int WAVES>
hipError_t launch_w(const lkv_ctx *c, const Plan &p, const void *Q, void *O, const int32_t *bt, int max_blocks,
                    const int32_t *cl, int num_seqs, Workspace ws, hipStream_t s) {
  launch_timed(c, true, p.num_parts == 1, paged_decode_kernel<T, D, G, WAVES>, dim3(c->cfg.num_kv_heads, num_seqs, p.num_parts),
                     dim3(WAVES * 64), s, (const T *)Q, (T *)O, c->pool, bt, max_blocks, cl, c->cfg.num_q_heads,
                     c->cfg.num_q_heads / c->cfg.num_kv_heads, c->block_bytes, (int)c->cfg.num_pool_blocks, c->scale, p.partition, p.num_parts, ws);
  return hipGetLastError();
}

template <int G, int WAVES, bool FP8>
hipError_t launch_mfma(const lkv_ctx *c, const Plan &p, const void *Q, void *O, const int32_t *bt, int max_blocks,
                       const int32_t *cl, int num_seqs, Workspace ws, hipStream_t s) {
  // one-dimensional grid: the even split's workgroups, or kv head fastest, then the rank of the (sequence,
  // partition) work item
  if ((int64_t)c->cfg.num_kv_heads * num_seqs * p.num_parts > INT32_MAX) return hipErrorInvalidValue;
  dim3 grid((unsigned)(p.even_wgs ? p.even_wgs : c->cfg.num_kv_heads * num_seqs * p.num_parts)), block(WAVES * 64);
  const int order = p.even_wgs ? kOrderEven : p.lpt ? kOrderLongest : kOrderPlain;
  launch_timed(c, true, p.num_parts == 1, paged_decode_mfma_kernel<G, WAVES, FP8>, grid, block, s, (const uint16_t *)Q,
                     (uint16_t *)O, c->pool, bt, max_blocks, cl, c->cfg.num_q_heads,
                     c->cfg.num_q_heads / c->cfg.num_kv_heads, c->block_bytes, (int)c->cfg.num_pool_blocks, FP8 ? c->scale * c->k_scale : c->scale, FP8 ? c->v_scale : 1.f,
                     p.partition, p.num_parts, num_seqs, order, ws);
  return hipGetLastError();
}

template <typename T, int D, int G>
hipError_t launch_t(const lkv_ctx *c, const void *Q, void *O, const int32_t *bt, int max_blocks, const int32_t *cl,
                    int num_seqs, float *wsbuf, hipStream_t s) {
  const Plan p = make_plan(c, num_seqs, max_blocks);
  if (num_seqs > 65535 || p.num_parts > 65535) return hipErrorInvalidValue;  // grid y and z limits
  const int Hq = c->cfg.num_q_heads;
  const int64_t entries = p.even_wgs ? ((int64_t)num_seqs * c->cfg.num_kv_heads + p.even_wgs) * (Hq / c->cfg.num_kv_heads)
                                     : (int64_t)num_seqs * Hq * p.num_parts;
  Workspace ws{wsbuf, wsbuf + entries * 2};
  hipError_t e;
  const bool fp8 = c->cfg.dtype == LKV_FP8_E4M3;
  if (p.mfma && sizeof(T) == 2 && D == 128) {  // make_plan sets mfma only for this case
    if (fp8)
      e = p.waves == 2 ? launch_mfma<G, 2, true>(c, p, Q, O, bt, max_blocks, cl, num_seqs, ws, s)
                       : launch_mfma<G, 8, true>(c, p, Q, O, bt, max_blocks, cl, num_seqs, ws, s);
    else
      e = p.waves == 2 ? launch_mfma<G, 2, false>(c, p, Q, O, bt, max_blocks, cl, num_seqs, ws, s)
                       : launch_mfma<G, 8, false>(c, p, Q, O, bt, max_blocks, cl, num_seqs, ws, s);
  } else if (fp8) {
    return hipErrorInvalidValue;  // 8-bit pools are only read by the kernel above (decode_supported says so)
  } else if constexpr (G <= 8) {
    e = launch_w<T, D, G, 4>(c, p, Q, O, bt, max_blocks, cl, num_seqs, ws, s);
  } else {
    return hipErrorInvalidValue;  // more than 8 heads per kv head only on the matrix-core kernel
  }
  if (e != hipSuccess || p.num_parts == 1) return e;
  if (p.even_wgs) {
    launch_timed(c, false, true, decode_combine_even_kernel<T, D>, dim3(num_seqs * Hq), dim3(D), s, (T *)O, cl,
                 max_blocks * kBlock, Hq, Hq / c->cfg.num_kv_heads, num_seqs, p.even_wgs, fp8 ? c->v_scale : 1.f, ws);
    return hipGetLastError();
  }
  launch_timed(c, false, true, decode_combine_kernel<T, D>, dim3(num_seqs * Hq), dim3(D), s, (T *)O, cl, max_blocks * kBlock, Hq,
                     p.partition,
                     p.num_parts, fp8 ? c->v_scale : 1.f, ws);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_g(const lkv_ctx *c, const void *Q, void *O, const int32_t *bt, int max_blocks, const int32_t *cl,
                    int num_seqs, float *ws, hipStream_t s) {
  const int group = c->cfg.num_q_heads / c->cfg.num_kv_heads;   // the smallest built capacity that holds it
  if (group == 1) return launch_t<T, D, 1>(c, Q, O, bt, max_blocks, cl, num_seqs, ws, s);
  if (group == 2) return launch_t<T, D, 2>(c, Q, O, bt, max_blocks, cl, num_seqs, ws, s);
  if (group <= 4) return launch_t<T, D, 4>(c, Q, O, bt, max_blocks, cl, num_seqs, ws, s);
  if (group <= 8) return launch_t<T, D, 8>(c, Q, O, bt, max_blocks, cl, num_seqs, ws, s);
  if (group <= 16) return launch_t<T, D, 16>(c, Q, O, bt, max_blocks, cl, num_seqs, ws, s);
  return hipErrorInvalidValue;
}

}  // namespace

namespace lkv {

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float *g_scratch_ptr[kMaxDevices] = {};
}  // namespace

hipError_t static_scratch_init(int device) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[device]) return hipSuccess;
  void *p = nullptr;
  const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));  // of the CURRENT device's copy
  if (e != hipSuccess) return e;
  g_scratch_ptr[device] = (float *)p;
  return hipSuccess;
}

float *static_scratch(int device) {
  if (device < 0 || device >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  return g_scratch_ptr[device];
}

bool decode_supported(const lkv_ctx *c) {
  const int g = c->cfg.num_q_heads / c->cfg.num_kv_heads;
  if (c->cfg.dtype == LKV_FP8_E4M3 && c->cfg.head_dim != 128) return false;
  // query heads per kv head: up to 16 on the matrix-core kernel (bf16 or 8-bit pool, head_dim 128), up to 8 otherwise
  const bool mfma = c->cfg.dtype != LKV_F32 && c->cfg.head_dim == 128;
  return c->cfg.block_size == kBlock && (c->cfg.head_dim == 64 || c->cfg.head_dim == 128) && g >= 1 &&
         g <= (mfma ? 16 : 8);
}

int64_t decode_workspace_bytes(const lkv_ctx *c, int32_t num_seqs, int32_t max_blocks) {
  const Plan p = make_plan(c, num_seqs, max_blocks);
  if (p.num_parts <= 1) return 0;
  const int64_t group = c->cfg.num_q_heads / c->cfg.num_kv_heads;
  const int64_t entries = p.even_wgs ? ((int64_t)num_seqs * c->cfg.num_kv_heads + p.even_wgs) * group
                                     : (int64_t)num_seqs * c->cfg.num_q_heads * p.num_parts;
  return entries * (2 + c->cfg.head_dim) * (int64_t)sizeof(float);
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
