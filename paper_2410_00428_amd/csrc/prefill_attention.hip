// Prefill attention over packed variable-length prompts (paper Section 2.1.1: all prompt tokens
// are processed in parallel; the attention cost is quadratic in the prompt length).
//
// bf16 path: the only dense contraction of the library, so it runs on the gfx950 matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulation).  A workgroup of four wavefronts owns 128
// consecutive queries of one (sequence, q head); each wavefront owns 32 of them and keeps its
// slice of Q in registers for the whole kernel.  Keys/values stream through LDS in tiles of 64.
// Scores are computed TRANSPOSED, S^T = K Q^T, so that after the MFMA every lane holds the
// scores of ONE query (its column) for 16 keys per 32-key block: the softmax row reductions are
// in-lane plus one exchange with the lane 32 away, and the exponentiated scores are already laid
// out as the B operand of the second product O^T = V^T P^T.  For that product the contraction
// index (key) of a lane's 8 elements is k(h,e) = 8*(e/4) + 4*h + e%4 within a 16-key slab; V is
// transposed on its way into LDS so the A operand reads those keys as two 8-byte words.
// Probabilities are rounded to bf16 for the second product; the row sum uses the fp32 values.
// Causal tiles above the diagonal are skipped, only tiles that touch it are masked.
//
// f32 path: plain fp32 vector arithmetic (sizes where this runs are launch-bound), one query per
// four lanes, keys/values through LDS.
#include "lkv_internal.hpp"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int BM = 128;  // queries per workgroup
constexpr int BN = 64;   // keys per tile
constexpr int kXcds = 8;
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 v = __builtin_convertvector(f, bf16x2);  // round to nearest even
  return __builtin_bit_cast(unsigned, v);
}

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(kThreads)
prefill_bf16_kernel(const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
                    uint16_t *__restrict__ O, const int32_t *__restrict__ cu_seqlens, int Hq, int Hkv,
                    int tiles_per_seq, int total_wgs, float scale_log2e) {
  constexpr int KS_STRIDE = D + 8;   // bf16 elements per K row in LDS (padding spreads rows over banks)
  constexpr int VT_STRIDE = BN + 4;  // bf16 elements per transposed-V row
  constexpr int OS_STRIDE = D + 8;
  constexpr int KK = D / 16;         // MFMA steps over the head dimension
  constexpr int DB = D / 32;         // 32-row blocks of O^T
  constexpr int KS_BYTES = BN * KS_STRIDE * 2, VT_BYTES = D * VT_STRIDE * 2;
  constexpr int OS_BYTES = 4 * 32 * OS_STRIDE * 2;
  constexpr int SMEM = (KS_BYTES + VT_BYTES) > OS_BYTES ? (KS_BYTES + VT_BYTES) : OS_BYTES;
  __shared__ __attribute__((aligned(16))) char smem[SMEM];
  char *Ks = smem, *Vt = smem + KS_BYTES;

  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of logical
  // tiles so the q tiles of one (sequence, head) share that XCD's L2.
  const int per_xcd = (total_wgs + kXcds - 1) / kXcds;
  const int logical = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
  if (logical >= total_wgs) return;
  const int qt = tiles_per_seq - 1 - logical % tiles_per_seq;  // heaviest (last) q tile first
  const int rest = logical / tiles_per_seq;
  const int h = rest % Hq, s = rest / Hq;
  const int t0 = cu_seqlens[s], n = cu_seqlens[s + 1] - t0;
  const int q0 = qt * BM;
  if (q0 >= n) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, ql = lane & 31, hh = lane >> 5;
  const int g = h / (Hq / Hkv);
  const int64_t q_stride = (int64_t)Hq * D, kv_stride = (int64_t)Hkv * D;
  const int wq0 = q0 + wave * 32;  // first query of this wavefront
  const int my_q = wq0 + ql;

  bf16x8 qreg[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    u32x4 w = {0, 0, 0, 0};
    if (my_q < n) w = *(const u32x4 *)(Q + (t0 + my_q) * q_stride + (int64_t)h * D + 16 * kk + 8 * hh);
    qreg[kk] = __builtin_bit_cast(bf16x8, w);
  }
  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
  float m = -INFINITY, lsum = 0.f;

  const int kv_end = CAUSAL ? min(n, q0 + BM) : n;
  const int ntiles = (kv_end + BN - 1) / BN;
  const uint16_t *Kg = K + (int64_t)t0 * kv_stride + (int64_t)g * D;
  const uint16_t *Vg = V + (int64_t)t0 * kv_stride + (int64_t)g * D;

  for (int j = 0; j < ntiles; ++j) {
    const int k0 = j * BN;
    __syncthreads();  // the previous tile's LDS reads are finished
    // K tile, row-major: 16 lanes per 2*D-byte row
    for (int p = tid; p < BN * (D / 8); p += kThreads) {
      const int row = p / (D / 8), pc = p % (D / 8);
      u32x4 w = {0, 0, 0, 0};
      if (k0 + row < n) w = *(const u32x4 *)(Kg + (int64_t)(k0 + row) * kv_stride + pc * 8);
      *(u32x4 *)(Ks + (row * KS_STRIDE + pc * 8) * 2) = w;
    }
    // V tile, transposed: a thread takes 4 keys x 8 channels and writes 8 channel rows of 4 keys
    for (int p = tid; p < (BN / 4) * (D / 8); p += kThreads) {
      const int kg = p / (D / 8), dg = p % (D / 8);
      u32x4 r[4];
#pragma unroll
      for (int kq = 0; kq < 4; ++kq) {
        r[kq] = u32x4{0, 0, 0, 0};
        if (k0 + 4 * kg + kq < n) r[kq] = *(const u32x4 *)(Vg + (int64_t)(k0 + 4 * kg + kq) * kv_stride + dg * 8);
      }
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        u32x2 even = {__builtin_amdgcn_perm(r[1][jj], r[0][jj], 0x05040100u),
                      __builtin_amdgcn_perm(r[3][jj], r[2][jj], 0x05040100u)};
        u32x2 odd = {__builtin_amdgcn_perm(r[1][jj], r[0][jj], 0x07060302u),
                     __builtin_amdgcn_perm(r[3][jj], r[2][jj], 0x07060302u)};
        *(u32x2 *)(Vt + ((8 * dg + 2 * jj) * VT_STRIDE + 4 * kg) * 2) = even;
        *(u32x2 *)(Vt + ((8 * dg + 2 * jj + 1) * VT_STRIDE + 4 * kg) * 2) = odd;
      }
    }
    __syncthreads();
    if (CAUSAL && k0 > wq0 + 31) continue;  // every key of the tile is after every query of this wavefront

    // S^T = K Q^T: rows = keys (two blocks of 32), columns = this wavefront's 32 queries
    f32x16 sacc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) sacc[kb][v] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        bf16x8 a = __builtin_bit_cast(bf16x8, *(const u32x4 *)(Ks + ((32 * kb + ql) * KS_STRIDE + 16 * kk + 8 * hh) * 2));
        sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[kk], sacc[kb], 0, 0, 0);
      }
    }
    // register v of a lane holds key 8*(v/4) + 4*hh + v%4 of the 32-key block
    const bool need_mask = (CAUSAL && k0 + BN - 1 > wq0) || (k0 + BN > n);
    if (need_mask) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = k0 + 32 * kb + 8 * (v / 4) + 4 * hh + (v % 4);
          if ((CAUSAL && key > my_q) || key >= n) sacc[kb][v] = -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sacc[kb][v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m, mx);
    const float ms = (m_new == -INFINITY ? 0.f : m_new) * scale_log2e;
    const float alpha = __builtin_amdgcn_exp2f(m * scale_log2e - ms);
    m = m_new;
    float psum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kb][v], scale_log2e, -ms));
        sacc[kb][v] = p;
        psum += p;
      }
    lsum = lsum * alpha + psum;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[db][v] *= alpha;

    // O^T += V^T P^T, 16 keys per step
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        u32x4 pw;
#pragma unroll
        for (int e = 0; e < 4; ++e) pw[e] = pack_bf16(sacc[kb][8 * half + 2 * e], sacc[kb][8 * half + 2 * e + 1]);
        const bf16x8 pb = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const char *vp = Vt + ((32 * db + ql) * VT_STRIDE + 32 * kb + 16 * half + 4 * hh) * 2;
          u32x2 lo = *(const u32x2 *)vp, hi = *(const u32x2 *)(vp + 16);
          u32x4 aw = {lo.x, lo.y, hi.x, hi.y};
          oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, aw), pb, oacc[db], 0, 0, 0);
        }
      }
  }

  lsum += __shfl_xor(lsum, 32);
  const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
  __syncthreads();  // K/V tiles are dead; reuse LDS to turn O^T into row-major rows
  char *Os = smem + wave * (32 * OS_STRIDE * 2);
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int d0 = 32 * db + 8 * q4 + 4 * hh;
      u32x2 w = {pack_bf16(oacc[db][4 * q4] * inv, oacc[db][4 * q4 + 1] * inv),
                 pack_bf16(oacc[db][4 * q4 + 2] * inv, oacc[db][4 * q4 + 3] * inv)};
      *(u32x2 *)(Os + (ql * OS_STRIDE + d0) * 2) = w;
    }
  __syncthreads();
  for (int p = lane; p < 32 * (D / 8); p += 64) {
    const int row = p / (D / 8), pc = p % (D / 8);
    if (wq0 + row < n)
      *(u32x4 *)(O + (t0 + wq0 + row) * q_stride + (int64_t)h * D + pc * 8) =
          *(const u32x4 *)(Os + (row * OS_STRIDE + pc * 8) * 2);
  }
}

// ------------------------------------------------------------------------------------------ f32
// 64 queries per workgroup, four lanes per query (each owns D/4 channels), 32-key tiles in LDS.
template <int D, bool CAUSAL>
__global__ void __launch_bounds__(kThreads)
prefill_f32_kernel(const float *__restrict__ Q, const float *__restrict__ K, const float *__restrict__ V,
                   float *__restrict__ O, const int32_t *__restrict__ cu_seqlens, int Hq, int Hkv, float scale) {
  constexpr int QB = 64, KB = 32, C = D / 4;
  __shared__ float Ks[KB][D + 4];
  __shared__ float Vs[KB][D + 4];
  const int s = blockIdx.z, h = blockIdx.y, q0 = blockIdx.x * QB;
  const int t0 = cu_seqlens[s], n = cu_seqlens[s + 1] - t0;
  if (q0 >= n) return;
  const int g = h / (Hq / Hkv);
  const int tid = threadIdx.x, qi = tid / 4, part = tid % 4;
  const int my_q = q0 + qi;
  const int64_t q_stride = (int64_t)Hq * D, kv_stride = (int64_t)Hkv * D;
  float q[C], acc[C];
#pragma unroll
  for (int c = 0; c < C; ++c) {
    q[c] = my_q < n ? Q[(t0 + my_q) * q_stride + (int64_t)h * D + part * C + c] * scale : 0.f;
    acc[c] = 0.f;
  }
  float m = -INFINITY, l = 0.f;
  const int kv_end = CAUSAL ? min(n, q0 + QB) : n;
  for (int k0 = 0; k0 < kv_end; k0 += KB) {
    __syncthreads();
    for (int p = tid; p < KB * D; p += kThreads) {
      const int row = p / D, col = p % D;
      const bool ok = k0 + row < n;
      const int64_t off = (int64_t)(t0 + k0 + row) * kv_stride + (int64_t)g * D + col;
      Ks[row][col] = ok ? K[off] : 0.f;
      Vs[row][col] = ok ? V[off] : 0.f;
    }
    __syncthreads();
    const int last = min(KB, kv_end - k0);
    for (int j = 0; j < last; ++j) {
      float d = 0.f;
#pragma unroll
      for (int c = 0; c < C; ++c) d = fmaf(q[c], Ks[j][part * C + c], d);
      d += __shfl_xor(d, 1);
      d += __shfl_xor(d, 2);
      const bool visible = CAUSAL ? (k0 + j <= my_q) : true;
      if (!visible) continue;  // lanes of a query agree; the shuffles above ran for all lanes
      const float m_new = fmaxf(m, d);
      const float alpha = expf(m - m_new), p = expf(d - m_new);
      l = l * alpha + p;
#pragma unroll
      for (int c = 0; c < C; ++c) acc[c] = fmaf(p, Vs[j][part * C + c], acc[c] * alpha);
      m = m_new;
    }
  }
  if (my_q < n) {
    const float inv = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
    for (int c = 0; c < C; ++c) O[(t0 + my_q) * q_stride + (int64_t)h * D + part * C + c] = acc[c] * inv;
  }
}

template <int D>
hipError_t launch_bf16(const lkv_ctx *c, const void *Q, const void *K, const void *V, void *O, const int32_t *cu,
                       int num_seqs, int max_seqlen, int causal, hipStream_t s) {
  const int tiles = (max_seqlen + BM - 1) / BM;
  const int64_t total = (int64_t)tiles * c->cfg.num_q_heads * num_seqs;
  if (total > INT32_MAX - kXcds) return hipErrorInvalidValue;
  const int per_xcd = (int)((total + kXcds - 1) / kXcds);
  const float sl2 = c->scale * kLog2e;
  dim3 grid((unsigned)(per_xcd * kXcds));
  if (causal)
    hipLaunchKernelGGL((prefill_bf16_kernel<D, true>), grid, dim3(kThreads), 0, s, (const uint16_t *)Q,
                       (const uint16_t *)K, (const uint16_t *)V, (uint16_t *)O, cu, c->cfg.num_q_heads,
                       c->cfg.num_kv_heads, tiles, (int)total, sl2);
  else
    hipLaunchKernelGGL((prefill_bf16_kernel<D, false>), grid, dim3(kThreads), 0, s, (const uint16_t *)Q,
                       (const uint16_t *)K, (const uint16_t *)V, (uint16_t *)O, cu, c->cfg.num_q_heads,
                       c->cfg.num_kv_heads, tiles, (int)total, sl2);
  return hipGetLastError();
}

template <int D>
hipError_t launch_f32(const lkv_ctx *c, const void *Q, const void *K, const void *V, void *O, const int32_t *cu,
                      int num_seqs, int max_seqlen, int causal, hipStream_t s) {
  dim3 grid((unsigned)((max_seqlen + 63) / 64), (unsigned)c->cfg.num_q_heads, (unsigned)num_seqs);
  if (causal)
    hipLaunchKernelGGL((prefill_f32_kernel<D, true>), grid, dim3(kThreads), 0, s, (const float *)Q, (const float *)K,
                       (const float *)V, (float *)O, cu, c->cfg.num_q_heads, c->cfg.num_kv_heads, c->scale);
  else
    hipLaunchKernelGGL((prefill_f32_kernel<D, false>), grid, dim3(kThreads), 0, s, (const float *)Q, (const float *)K,
                       (const float *)V, (float *)O, cu, c->cfg.num_q_heads, c->cfg.num_kv_heads, c->scale);
  return hipGetLastError();
}

}  // namespace

namespace lkv {

bool prefill_supported(const lkv_ctx *c) { return c->cfg.head_dim == 64 || c->cfg.head_dim == 128; }

hipError_t launch_prefill(const lkv_ctx *c, const void *Q, const void *K, const void *V, void *O, const int32_t *cu,
                          int32_t num_seqs, int32_t max_seqlen, int32_t causal, hipStream_t s) {
  if (c->cfg.num_q_heads > 65535 || num_seqs > 65535) return hipErrorInvalidValue;
  if (c->cfg.dtype == LKV_F32)
    return c->cfg.head_dim == 64 ? launch_f32<64>(c, Q, K, V, O, cu, num_seqs, max_seqlen, causal, s)
                                 : launch_f32<128>(c, Q, K, V, O, cu, num_seqs, max_seqlen, causal, s);
  return c->cfg.head_dim == 64 ? launch_bf16<64>(c, Q, K, V, O, cu, num_seqs, max_seqlen, causal, s)
                               : launch_bf16<128>(c, Q, K, V, O, cu, num_seqs, max_seqlen, causal, s);
}

}  // namespace lkv
