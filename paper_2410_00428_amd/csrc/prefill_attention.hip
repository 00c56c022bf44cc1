// Prefill attention over packed variable-length prompts (paper Section 2.1.1: all prompt tokens
// are processed in parallel; the attention cost is quadratic in the prompt length).
//
// bf16, head_dim 128 (the shape of every bf16 workload): the only dense contraction of the library, so it runs
// on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation).  A workgroup of four wavefronts owns
// 128 consecutive queries of one (sequence, q head); each wavefront owns 32 of them and keeps its slice of Q in
// registers.  Keys and values stream through LDS in units of 32 keys:
//   * global -> LDS goes through `buffer_load_dwordx4 ... lds` (no registers, no LDS store instructions); a
//     unit is stored row-major, its 16-byte pieces XOR-swizzled so that every operand read is bank-conflict
//     free; four units of K and four of V are in flight or in use at any time (64 KiB, two workgroups per CU);
//   * scores are computed TRANSPOSED, S^T = K Q^T, so that after the MFMA every lane holds the scores of ONE
//     query (its column) for 16 of the 32 keys: the softmax row reductions are in-lane plus one
//     v_permlane32_swap, and the exponentiated scores are already laid out as the B operand of the second
//     product O^T = V^T P^T;
//   * the A operand of that product is V^T, which is read straight out of the row-major unit with the
//     transposing LDS load ds_read_b64_tr_b16;
//   * the loop is software-pipelined over units: the score MFMAs of unit u+1 are issued before the softmax of
//     unit u, and the first operands of unit u+2 are fetched from LDS before the barrier that ends unit u.
// Probabilities are rounded to bf16 for the second product; the row sum uses the fp32 values.  Under the causal
// mask a workgroup handles query tile T-1-p and then tile p of its head, whose key ranges add up to the same
// length for every p: all workgroups of a launch cost the same.  Units above the diagonal are skipped, only
// the unit that touches it is masked.
//
// bf16, head_dim 64: the earlier register-staged kernel (64-key tiles, V transposed on its way into LDS).
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
constexpr int BN = 64;   // keys per tile
constexpr int kXcds = 8;
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 v = __builtin_convertvector(f, bf16x2);  // round to nearest even
  return __builtin_bit_cast(unsigned, v);
}

// Sequence s of the batch as the kernels use it: tokens t0 .. t0 + n - 1 of the packed tensors.  cu_seqlens lives in
// device memory, where the host cannot check it; whatever it holds, 0 <= t0, 0 <= n <= max_seqlen and
// t0 + n <= total_tokens come out of here, so that no row outside Q, K, V and O is ever addressed (a wrong entry gives
// wrong or unwritten rows, not a fault).
__device__ __forceinline__ void seq_range(const int32_t *__restrict__ cu_seqlens, int s, int total_tokens, int max_seqlen,
                                          int &t0, int &n) {
  const int a = min(max(cu_seqlens[s], 0), total_tokens);
  const int b = min(max(cu_seqlens[s + 1], a), total_tokens);
  t0 = a;
  n = min(b - a, max_seqlen);
}
__device__ __forceinline__ int seq_len(const int32_t *__restrict__ cu_seqlens, int s, int total_tokens, int max_seqlen) {
  int t0, n;
  seq_range(cu_seqlens, s, total_tokens, max_seqlen, t0, n);
  return n;
}

// Work slot k of a head -> (sequence, index of the tile pair inside it).  A sequence of n tokens owns ceil(n / 256)
// consecutive slots (one per pair of 128-query tiles).  Up to 64 sequences are taken LONGEST FIRST (ties in batch
// order), so that the long workgroups of an unequal batch start first and the short ones fill the end of the launch;
// larger batches keep the batch order.  Every wavefront rebuilds the list from cu_seqlens.  Returns false when k is
// past the last slot.
__device__ __forceinline__ bool find_pair_slot(const int32_t *__restrict__ cu_seqlens, int num_seqs, int total_tokens,
                                               int max_seqlen, int k, int lane, int &seq, int &pidx) {
  if (num_seqs <= 64) {
    const int cnt = lane < num_seqs ? (seq_len(cu_seqlens, lane, total_tokens, max_seqlen) + 255) / 256 : 0;
    int pos = 0;  // slots of the sequences that come before this lane's in the longest-first order
    for (int t = 0; t < num_seqs; ++t) {
      const int ct = __builtin_amdgcn_readlane(cnt, t);
      pos += (ct > cnt || (ct == cnt && t < lane)) ? ct : 0;
    }
    const unsigned long long mask = __ballot(k >= pos && k < pos + cnt);
    if (mask == 0) return false;
    const int src = __ffsll((long long)mask) - 1;
    seq = src;
    pidx = k - __builtin_amdgcn_readlane(pos, src);
    return true;
  }
  int base = 0;
  for (int s0 = 0; s0 < num_seqs; s0 += 64) {
    const int s = s0 + lane;
    const int cnt = s < num_seqs ? (seq_len(cu_seqlens, s, total_tokens, max_seqlen) + 255) / 256 : 0;
    int inc = cnt;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int t = __shfl_up(inc, d);
      if (lane >= d) inc += t;
    }
    const int total = __builtin_amdgcn_readlane(inc, 63);
    if (k < base + total) {
      const unsigned long long mask = __ballot(base + inc > k);
      const int src = __ffsll((long long)mask) - 1;
      seq = s0 + src;
      pidx = k - base - __builtin_amdgcn_readlane(inc - cnt, src);
      return true;
    }
    base += total;
  }
  return false;
}
// QB blocks of 32 queries per wavefront (each K / V^T operand read from LDS feeds QB MFMAs; QB = 1 keeps
// the kernel within 256 registers so that two workgroups share a CU and hide each other's latencies).
// LDS is double-buffered: the next tile's global loads are issued before the current tile's math and
// parked in registers until it is done, so there is one barrier per tile.
template <int D, bool CAUSAL, int QB>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
prefill_bf16_kernel(const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
                     uint16_t *__restrict__ O, const int32_t *__restrict__ cu_seqlens, int Hq, int Hkv,
                     int tiles_per_seq, int total_wgs, int total_tokens, int max_seqlen, float scale_log2e) {
  constexpr int WQ = 32 * QB;        // queries per wavefront
  constexpr int BMQ = 4 * WQ;        // queries per workgroup
  constexpr int KS_STRIDE = D + 8, VT_STRIDE = BN + 4, OS_STRIDE = D + 8;
  constexpr int KK = D / 16, DB = D / 32;
  constexpr int KS_BYTES = BN * KS_STRIDE * 2, VT_BYTES = D * VT_STRIDE * 2;
  constexpr int BUF_BYTES = KS_BYTES + VT_BYTES;
  constexpr int OS_BYTES = 4 * WQ * OS_STRIDE * 2;
  constexpr int SMEM = 2 * BUF_BYTES > OS_BYTES ? 2 * BUF_BYTES : OS_BYTES;
  constexpr int KPIECES = BN * (D / 8), VPATCHES = (BN / 4) * (D / 8);
  constexpr int KP = (KPIECES + kThreads - 1) / kThreads;    // 16-byte K pieces per thread per tile
  constexpr int VP = (VPATCHES + kThreads - 1) / kThreads;   // 4-key x 8-channel V patches per thread per tile
  __shared__ __attribute__((aligned(16))) char smem[SMEM];

  // workgroup order: (sequence, head) pairs in turn, each with its query tiles longest first; consecutive
  // workgroups go to consecutive XCDs, so the load is even whatever the head count
  if ((int)blockIdx.x >= total_wgs) return;
  const int qt = tiles_per_seq - 1 - blockIdx.x % tiles_per_seq;
  const int rest = blockIdx.x / tiles_per_seq;
  const int h = rest % Hq, s = rest / Hq;
  int t0, n;
  seq_range(cu_seqlens, s, total_tokens, max_seqlen, t0, n);
  const int q0 = qt * BMQ;
  if (q0 >= n) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, ql = lane & 31, hh = lane >> 5;
  const int g = h / (Hq / Hkv);
  const int64_t q_stride = (int64_t)Hq * D, kv_stride = (int64_t)Hkv * D;
  const int wq0 = q0 + wave * WQ;

  bf16x8 qreg[QB][KK];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const int q = min(wq0 + 32 * qb + ql, n - 1);  // rows past the end compute on a copy and are not stored
      const u32x4 w = *(const u32x4 *)(Q + (t0 + q) * q_stride + (int64_t)h * D + 16 * kk + 8 * hh);
      qreg[qb][kk] = __builtin_bit_cast(bf16x8, w);
    }
  f32x16 oacc[QB][DB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[qb][db][v] = 0.f;
  float m[QB], lsum[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m[qb] = -INFINITY;
    lsum[qb] = 0.f;
  }

  const int kv_end = CAUSAL ? min(n, q0 + BMQ) : n;
  const int ntiles = (kv_end + BN - 1) / BN;
  const uint16_t *Kg = K + (int64_t)t0 * kv_stride + (int64_t)g * D;
  const uint16_t *Vg = V + (int64_t)t0 * kv_stride + (int64_t)g * D;

  // Global loads of a tile go through buffer descriptors that end with the sequence's last row: the
  // address is a scalar tile offset plus a per-lane byte offset that never changes (no address arithmetic
  // in the loop), and rows past the end of the sequence read as zeros without any branch.
  u32x4 kreg[KP], vreg[VP][4];
  unsigned koff[KP], voff[VP][4];
  const unsigned row_bytes = (unsigned)kv_stride * 2;
  const unsigned extent = (unsigned)(n - 1) * row_bytes + D * 2;
  const __amdgpu_buffer_rsrc_t krsrc = __builtin_amdgcn_make_buffer_rsrc((void *)Kg, 0, extent, 0x00020000);
  const __amdgpu_buffer_rsrc_t vrsrc = __builtin_amdgcn_make_buffer_rsrc((void *)Vg, 0, extent, 0x00020000);
#pragma unroll
  for (int i = 0; i < KP; ++i) {
    const int p = tid + i * kThreads;
    koff[i] = (unsigned)(p / (D / 8)) * row_bytes + (p % (D / 8)) * 16;
  }
#pragma unroll
  for (int i = 0; i < VP; ++i) {
    const int p = tid + i * kThreads;
#pragma unroll
    for (int kq = 0; kq < 4; ++kq) voff[i][kq] = (unsigned)(4 * (p / (D / 8)) + kq) * row_bytes + (p % (D / 8)) * 16;
  }
  auto gload = [&](int k0) {
    const unsigned soff = (unsigned)k0 * row_bytes;
#pragma unroll
    for (int i = 0; i < KP; ++i)
      if (KPIECES % kThreads == 0 || tid + i * kThreads < KPIECES)
        kreg[i] = __builtin_amdgcn_raw_buffer_load_b128(krsrc, koff[i], soff, 0);
#pragma unroll
    for (int i = 0; i < VP; ++i)
#pragma unroll
      for (int kq = 0; kq < 4; ++kq)
        if (VPATCHES % kThreads == 0 || tid + i * kThreads < VPATCHES)
          vreg[i][kq] = __builtin_amdgcn_raw_buffer_load_b128(vrsrc, voff[i][kq], soff, 0);
  };
  auto lstore = [&](char *buf) {
    char *Ks = buf, *Vt = buf + KS_BYTES;
#pragma unroll
    for (int i = 0; i < KP; ++i) {
      const int p = tid + i * kThreads, row = p / (D / 8), pc = p % (D / 8);
      if (KPIECES % kThreads == 0 || p < KPIECES) *(u32x4 *)(Ks + (row * KS_STRIDE + pc * 8) * 2) = kreg[i];
    }
#pragma unroll
    for (int i = 0; i < VP; ++i) {
      const int p = tid + i * kThreads, kg = p / (D / 8), dg = p % (D / 8);
      if (VPATCHES % kThreads != 0 && p >= VPATCHES) continue;
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        u32x2 even = {__builtin_amdgcn_perm(vreg[i][1][jj], vreg[i][0][jj], 0x05040100u),
                      __builtin_amdgcn_perm(vreg[i][3][jj], vreg[i][2][jj], 0x05040100u)};
        u32x2 odd = {__builtin_amdgcn_perm(vreg[i][1][jj], vreg[i][0][jj], 0x07060302u),
                     __builtin_amdgcn_perm(vreg[i][3][jj], vreg[i][2][jj], 0x07060302u)};
        // 8-byte column units are XOR-swizzled with bits of the row so that the 16 lanes of a write
        // (rows 8 apart) and the 16 lanes of an operand read (consecutive rows) each cover all banks
        const int unit = kg ^ ((dg >> 1) & 7);
        *(u32x2 *)(Vt + (8 * dg + 2 * jj) * (VT_STRIDE * 2) + unit * 8) = even;
        *(u32x2 *)(Vt + (8 * dg + 2 * jj + 1) * (VT_STRIDE * 2) + unit * 8) = odd;
      }
    }
  };

  gload(0);
  lstore(smem);
  // Pin the Q loads in front of the loop.  The compiler would otherwise sink them behind the barrier, and
  // because memory-wait counters are in-order, every first use of Q inside the loop would then also wait
  // for the prefetch loads issued in the same iteration, which defeats the prefetch.
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) asm volatile("" : "+v"(qreg[qb][kk]));
  __syncthreads();

  for (int j = 0; j < ntiles; ++j) {
    const int k0 = j * BN;
    const char *Ks = smem + (j & 1) * BUF_BYTES, *Vt = Ks + KS_BYTES;
    if (j + 1 < ntiles) gload(k0 + BN);

    if (!(CAUSAL && k0 > wq0 + WQ - 1)) {
      f32x16 sacc[QB][2];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) sacc[qb][kb][v] = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          const bf16x8 a =
              __builtin_bit_cast(bf16x8, *(const u32x4 *)(Ks + ((32 * kb + ql) * KS_STRIDE + 16 * kk + 8 * hh) * 2));
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            sacc[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[qb][kk], sacc[qb][kb], 0, 0, 0);
        }
      const bool need_mask = (CAUSAL && k0 + BN - 1 > wq0) || (k0 + BN > n);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const int my_q = wq0 + 32 * qb + ql;
        if (need_mask) {
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int key = k0 + 32 * kb + 8 * (v / 4) + 4 * hh + (v % 4);
              if ((CAUSAL && key > my_q) || key >= n) sacc[qb][kb][v] = -INFINITY;
            }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sacc[qb][kb][v]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m[qb], mx);
        const float ms = (m_new == -INFINITY ? 0.f : m_new) * scale_log2e;
        const float alpha = __builtin_amdgcn_exp2f(m[qb] * scale_log2e - ms);
        const bool grew = m_new > m[qb];
        m[qb] = m_new;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const float p = __builtin_amdgcn_exp2f(fmaf(sacc[qb][kb][v], scale_log2e, -ms));
            sacc[qb][kb][v] = p;
            psum += p;
          }
        lsum[qb] = lsum[qb] * alpha + psum;
        if (__any(grew)) {  // once the running maxima have settled the accumulators need no rescaling
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[qb][db][v] *= alpha;
        }
      }
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          bf16x8 pb[QB];
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) {
            u32x4 pw;
#pragma unroll
            for (int e = 0; e < 4; ++e)
              pw[e] = pack_bf16(sacc[qb][kb][8 * half + 2 * e], sacc[qb][kb][8 * half + 2 * e + 1]);
            pb[qb] = __builtin_bit_cast(bf16x8, pw);
          }
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            const int sw = (2 * db + (ql >> 4)) & 7, unit = 8 * kb + 4 * half + hh;
            const char *vrow = Vt + (32 * db + ql) * (VT_STRIDE * 2);
            const u32x2 lo = *(const u32x2 *)(vrow + ((unit ^ sw) * 8)), hi = *(const u32x2 *)(vrow + (((unit + 2) ^ sw) * 8));
            const bf16x8 a = __builtin_bit_cast(bf16x8, u32x4{lo.x, lo.y, hi.x, hi.y});
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
              oacc[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[qb], oacc[qb][db], 0, 0, 0);
          }
        }
    }
    if (j + 1 < ntiles) lstore(smem + ((j + 1) & 1) * BUF_BYTES);
    __syncthreads();
  }

  // K/V tiles are dead (the loop ended on a barrier); reuse LDS to turn O^T into row-major rows
  char *Os = smem + wave * (WQ * OS_STRIDE * 2);
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    float l = lsum[qb];
    l += __shfl_xor(l, 32);
    const float inv = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int d0 = 32 * db + 8 * q4 + 4 * hh;
        u32x2 w = {pack_bf16(oacc[qb][db][4 * q4] * inv, oacc[qb][db][4 * q4 + 1] * inv),
                   pack_bf16(oacc[qb][db][4 * q4 + 2] * inv, oacc[qb][db][4 * q4 + 3] * inv)};
        *(u32x2 *)(Os + ((32 * qb + ql) * OS_STRIDE + d0) * 2) = w;
      }
  }
  __syncthreads();
  for (int p = lane; p < WQ * (D / 8); p += 64) {
    const int row = p / (D / 8), pc = p % (D / 8);
    if (wq0 + row < n)
      *(u32x4 *)(O + (t0 + wq0 + row) * q_stride + (int64_t)h * D + pc * 8) =
          *(const u32x4 *)(Os + (row * OS_STRIDE + pc * 8) * 2);
  }
}

// ------------------------------------------------------------------------------------------ bf16, d = 128
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// max / sum of a value and the value held by the lane 32 away (same result in both lanes)
__device__ __forceinline__ float both_max(float x) {
  auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}
__device__ __forceinline__ float both_sum(float x) {
  auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
}

// 16 bytes per lane from a buffer straight into LDS at lds_addr + lane*16 (lds_addr is wave-uniform).  Issued
// through inline asm so that the compiler does not tie later LDS reads to these loads: the kernel waits for them
// explicitly (vmcnt) before the barrier that publishes a unit.
// (m0 carries the LDS address of such a load; the compiler itself never keeps a value in m0 in this file)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, unsigned lds_addr, unsigned voffset, unsigned soffset) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset)
               : "memory", "m0");
}
#pragma clang diagnostic pop
constexpr int kVmcnt0 = 0x0F70;  // s_waitcnt vmcnt(0), other counters untouched
constexpr int kVmcnt6 = 0x0F76;  // s_waitcnt vmcnt(6)

template <bool CAUSAL>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
prefill_bf16_d128_kernel(const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
                         uint16_t *__restrict__ O, const int32_t *__restrict__ cu_seqlens, int Hq, int Hkv,
                         int num_seqs, int xcd_heads, int total_tokens, int max_seqlen, float scale_log2e) {
  constexpr int D = 128, UK = 32, KR = 4, VR = 4, TB = UK * D * 2, VOFF = KR * TB;
  constexpr int BMQ = 128, WQ = 32, OS_STRIDE = D + 8;
  __shared__ __attribute__((aligned(1024))) char smem[(KR + VR) * TB];

  // Workgroup order.  A workgroup takes tile T-1-p and then tile p of a (sequence, head) pair: equal cost for all
  // p of a sequence.  The grid holds, per query head, `slots` work slots, an upper bound of the batch's tile pairs
  // derived on the host from the total token count; find_pair_slot turns a slot into (sequence, p), longest
  // sequences first, so a batch of unequal sequences launches about as many workgroups as it has tile pairs and its
  // long workgroups start first.  Slot-major order: all heads take slot 0, then slot 1, ...
  //  * xcd_heads != 0 (the number of kv heads is a multiple of 8): XCD x (= blockIdx.x % 8) owns kv heads x, x+8,
  //    ... of every sequence, so all tiles of a kv group share one L2 and every XCD is loaded alike.
  //  * otherwise workgroup b is simply (slot b / Hq, head b % Hq): balanced for any head count (a tensor-parallel
  //    slice may have one kv head), at the price of a head's K/V passing through several L2s.
  const int lane = threadIdx.x & 63;
  int h, k;
  if (xcd_heads) {
    const int xcd = blockIdx.x % kXcds, li = blockIdx.x / kXcds;
    const int G = Hq / Hkv, hpx = Hq / kXcds, lhead = li % hpx;
    h = ((lhead / G) * kXcds + xcd) * G + lhead % G;
    k = li / hpx;
  } else {
    h = blockIdx.x % Hq;
    k = blockIdx.x / Hq;
  }
  int s, pidx;
  if (!find_pair_slot(cu_seqlens, num_seqs, total_tokens, max_seqlen, k, lane, s, pidx)) return;
  int t0, n;
  seq_range(cu_seqlens, s, total_tokens, max_seqlen, t0, n);
  const int tiles_per_seq = (n + BMQ - 1) / BMQ;

  const int tid = threadIdx.x, ql = lane & 31, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = h / (Hq / Hkv);
  const int64_t q_stride = (int64_t)Hq * D, kv_stride = (int64_t)Hkv * D;

  // ---- global -> LDS: wave w fills chunks 2w and 2w+1 (4 rows of 256 B each) of every unit.  Lane L of a chunk
  // writes LDS slot L%16 of row L/16; it fetches the piece that the swizzle assigns to that slot.
  const unsigned row_bytes = (unsigned)kv_stride * 2;
  const unsigned extent = (unsigned)(n - 1) * row_bytes + D * 2;
  const __amdgpu_buffer_rsrc_t krsrc =
      __builtin_amdgcn_make_buffer_rsrc((void *)(K + (int64_t)t0 * kv_stride + (int64_t)g * D), 0, extent, 0x00020000);
  const __amdgpu_buffer_rsrc_t vrsrc =
      __builtin_amdgcn_make_buffer_rsrc((void *)(V + (int64_t)t0 * kv_stride + (int64_t)g * D), 0, extent, 0x00020000);
  const int lslot = lane & 15;
  const unsigned wave_lds = (unsigned)(2 * wave * 1024);
  unsigned koff[2], voff[2];
  int lrow[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int r = 4 * (2 * wave + i) + (lane >> 4);
    lrow[i] = r;
    koff[i] = (unsigned)r * row_bytes + (unsigned)((lslot ^ (r & 15)) * 16);         // K: piece p of row r at slot p ^ (r % 16)
    voff[i] = (unsigned)r * row_bytes + (unsigned)((lslot ^ ((r & 3) << 2)) * 16);   // V: 64-byte groups rotated by r % 4
  }
  // ---- LDS operand addresses (slot 0 of each ring)
  unsigned kaddr[8], vaddr[4];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) kaddr[kk] = (unsigned)(ql * 256 + (((2 * kk + hh) ^ (ql & 15)) << 4));
  {
    // ds_read_b64_tr_b16: within 16 lanes, result lane i element j = element i%4 of the 8 bytes addressed by lane
    // 4j + i/4.  Source lane s16 therefore points at key row (s16/4), channels 4*(s16%4).. of its 16-channel block.
    const int s16 = lane & 15, dhalf = (lane >> 4) & 1;
#pragma unroll
    for (int db = 0; db < 4; ++db)
      vaddr[db] = (unsigned)(VOFF + (4 * hh + (s16 >> 2)) * 256 + ((db ^ (s16 >> 2)) * 64) + (2 * dhalf + ((s16 & 3) >> 1)) * 16 +
                             (s16 & 1) * 8);
  }
  lds_char *lds = (lds_char *)smem;
  auto kread = [&](int slot_off, int kk) -> bf16x8 {
    return __builtin_bit_cast(bf16x8, *(const u32x4 *)(smem + slot_off + kaddr[kk]));
  };
  // A operand of O^T += V^T P^T for channel block db and 16-key slab sl of the unit in the given V ring slot
  auto vread = [&](int slot_off, int sl, int db) -> bf16x8 {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(lds + slot_off + vaddr[db] + sl * 16 * 256));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(lds + slot_off + vaddr[db] + (sl * 16 + 8) * 256));
    const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
    return __builtin_bit_cast(bf16x8, u32x4{l2.x, l2.y, h2.x, h2.y});
  };

  for (int rep = 0; rep < 2; ++rep) {
    const int qt = rep == 0 ? tiles_per_seq - 1 - pidx : pidx;
    if (rep == 1 && 2 * pidx == tiles_per_seq - 1) break;
    const int q0 = qt * BMQ;
    if (q0 >= n) continue;
    if (rep == 1) __syncthreads();  // the first tile's output staging in LDS has been read

    const int wq0 = q0 + wave * WQ;
    const int my_q = wq0 + ql;
    bf16x8 qreg[8];
    {
      const int q = min(my_q, n - 1);  // rows past the end compute on a copy and are not stored
      const uint16_t *qp = Q + (t0 + q) * q_stride + (int64_t)h * D + 8 * hh;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) qreg[kk] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(qp + 16 * kk));
    }
    const int kv_end = CAUSAL ? min(n, q0 + BMQ) : n;
    const int nunits = (kv_end + UK - 1) / UK;
    // last unit this wavefront needs; none at all when its 32 rows lie past the end of the sequence
    const int last_w = wq0 >= n ? -1 : CAUSAL ? min(nunits - 1, wq0 / UK) : nunits - 1;

    // rows past the end of the sequence are fetched as copies of the last row (their scores are masked)
    auto issue = [&](const __amdgpu_buffer_rsrc_t &rsrc, const unsigned (&off)[2], int t, unsigned ring_base, bool is_k) {
      if (t >= nunits) return;
      const int k0 = t * UK;
      const unsigned soff = (unsigned)k0 * row_bytes;
      const unsigned dst = ring_base + (unsigned)((t % 4) * TB) + wave_lds;
      if (k0 + UK <= n) {
        dma16(rsrc, dst, off[0], soff);
        dma16(rsrc, dst + 1024, off[1], soff);
      } else {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          const int rr = min(lrow[i], n - 1 - k0);
          const int sw = is_k ? (lrow[i] & 15) : ((lrow[i] & 3) << 2);
          dma16(rsrc, dst + i * 1024, (unsigned)rr * row_bytes + (unsigned)((lslot ^ sw) * 16), soff);
        }
      }
    };
    auto issue_k = [&](int t) { issue(krsrc, koff, t, 0u, true); };
    auto issue_v = [&](int t) { issue(vrsrc, voff, t, (unsigned)VOFF, false); };

    f32x16 oacc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
    float m = -INFINITY, lsum = 0.f;

    // ---- prologue: fill the rings, scores of unit 0, first operands of unit 1
    issue_k(0);
    issue_k(1);
    issue_v(0);
    issue_k(2);
    issue_v(1);
    issue_k(3);
    issue_v(2);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) asm volatile("" : "+v"(qreg[kk]));
    __builtin_amdgcn_s_waitcnt(kVmcnt0);
    __syncthreads();

    f32x16 s_a, s_b;
#pragma unroll
    for (int v = 0; v < 16; ++v) s_a[v] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) s_a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kread(0, kk), qreg[kk], s_a, 0, 0, 0);
    bf16x8 ka[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) ka[kk] = kread(TB, kk);

    // softmax of one unit's scores: probabilities (bf16, B-operand layout of the second product), reference
    // maximum / sum
    constexpr float kLazy = 8.f;
    auto softmax = [&](f32x16 &sc, bf16x8 (&pb)[2], bool need_mask, int k0) {
      if (need_mask) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = k0 + 8 * (v / 4) + 4 * hh + (v % 4);
          if ((CAUSAL && key > my_q) || key >= n) sc[v] = -INFINITY;
        }
      }
      float mx = fmaxf(sc[0], sc[1]);
#pragma unroll
      for (int v = 2; v < 16; ++v) mx = fmaxf(mx, sc[v]);
      mx = both_max(mx);
      // m is the REFERENCE of the exponentials, in scaled log2 units.  It follows the running maximum lazily: it
      // only moves when a score exceeds it by more than kLazy, so probabilities stay below 2^kLazy (exact in
      // fp32 sums and as bf16 operands: both keep their relative precision at that magnitude) and the 64 output
      // accumulators are rescaled a few times per row instead of whenever any of a wavefront's 32 running maxima
      // grows (three units out of four at 2048 keys).  The quotient O / l does not depend on the reference.
      const float mxs = mx * scale_log2e;
      const bool grew = mxs > m + kLazy;
      if (__any(grew)) {
        const float alpha = grew ? __builtin_amdgcn_exp2f(m - mxs) : 1.f;  // m = -inf on first use: 0
        m = grew ? mxs : m;
        lsum *= alpha;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int v = 0; v < 16; ++v) oacc[db][v] *= alpha;
      }
      const float ms = m == -INFINITY ? 0.f : m;  // a row that has seen no key yet: exp2(-inf - 0) = 0
      float psum = 0.f;
      float p[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        p[v] = __builtin_amdgcn_exp2f(fmaf(sc[v], scale_log2e, -ms));
        psum += p[v];
      }
      lsum += psum;
#pragma unroll
      for (int sl = 0; sl < 2; ++sl) {
        u32x4 pw;
#pragma unroll
        for (int e = 0; e < 4; ++e) pw[e] = pack_bf16(p[8 * sl + 2 * e], p[8 * sl + 2 * e + 1]);
        pb[sl] = __builtin_bit_cast(bf16x8, pw);
      }
    };

    // One fully visible unit u (u % 4 == I) that is followed by a unit every wavefront of the workgroup needs.
    // Ring slots are compile-time constants.  Loads issued here: K of unit u+4 (into the slot unit u left after
    // the previous barrier) and V of unit u+3.  At the closing barrier K of unit u+3 and V of unit u+1 must have
    // landed: everything but the six most recent loads (V u+2, K u+4, V u+3).
#define LKV_UNIT(I, S_IN, S_OUT)                                                                                   \
  {                                                                                                                \
    constexpr int KS1 = ((I + 1) % KR) * TB, KS2 = ((I + 2) % KR) * TB, VS = (I % VR) * TB;                         \
    {                                                                                                              \
      const unsigned so_k = (unsigned)((u + I + 4) * UK) * row_bytes, so_v = (unsigned)((u + I + 3) * UK) * row_bytes; \
      constexpr unsigned DK = (I % KR) * TB, DV = VOFF + ((I + 3) % VR) * TB;                                      \
      dma16(krsrc, DK + wave_lds, koff[0], so_k);                                                                  \
      dma16(krsrc, DK + wave_lds + 1024, koff[1], so_k);                                                           \
      dma16(vrsrc, DV + wave_lds, voff[0], so_v);                                                                  \
      dma16(vrsrc, DV + wave_lds + 1024, voff[1], so_v);                                                           \
    }                                                                                                              \
    bf16x8 kb[4], va[4], vb[4], pb[2];                                                                             \
    _Pragma("unroll") for (int kk = 0; kk < 4; ++kk) kb[kk] = kread(KS1, 4 + kk);                                   \
    _Pragma("unroll") for (int db = 0; db < 4; ++db) va[db] = vread(VS, 0, db);                                     \
    _Pragma("unroll") for (int v = 0; v < 16; ++v) S_OUT[v] = 0.f;                                                  \
    _Pragma("unroll") for (int kk = 0; kk < 4; ++kk)                                                                \
        S_OUT = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk], qreg[kk], S_OUT, 0, 0, 0);                          \
    _Pragma("unroll") for (int kk = 0; kk < 4; ++kk)                                                                \
        S_OUT = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kb[kk], qreg[4 + kk], S_OUT, 0, 0, 0);                      \
    softmax(S_IN, pb, false, 0);                                                                                   \
    _Pragma("unroll") for (int db = 0; db < 4; ++db) vb[db] = vread(VS, 1, db);                                     \
    _Pragma("unroll") for (int kk = 0; kk < 4; ++kk) ka[kk] = kread(KS2, kk);                                       \
    _Pragma("unroll") for (int db = 0; db < 4; ++db)                                                                \
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[db], pb[0], oacc[db], 0, 0, 0);                       \
    _Pragma("unroll") for (int db = 0; db < 4; ++db)                                                                \
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vb[db], pb[1], oacc[db], 0, 0, 0);                       \
    __builtin_amdgcn_s_waitcnt(kVmcnt6);                                                                           \
    __syncthreads();                                                                                               \
  }

    // units below u_main are fully visible to all four wavefronts and are followed by a unit that all of them
    // need; inside the unrolled loop every unit that is fetched is a complete one (no row clamping)
    const int u_main = CAUSAL ? min(q0, n) / UK : (n / UK - 1);
    const int full_units = n / UK;
    int u = 0;
    for (; u + 4 <= u_main && u + 8 <= min(nunits, full_units); u += 4) {
      LKV_UNIT(0, s_a, s_b)
      LKV_UNIT(1, s_b, s_a)
      LKV_UNIT(2, s_a, s_b)
      LKV_UNIT(3, s_b, s_a)
    }
#undef LKV_UNIT
    // remaining units: masks, wavefronts that run out of visible keys, ring slots computed at run time.  The last
    // loads are issued in iteration nunits-4; after that iteration's barrier every unit is in LDS and none is
    // overwritten any more, so the wavefronts finish their remaining units without synchronising.
    f32x16 s_cur = s_a;
    const int u_sync_last = max(u, nunits - 4);
    for (; u < nunits; ++u) {
      issue_k(u + 4);
      issue_v(u + 3);
      if (u <= last_w) {
        const int kslot_n = ((u + 1) % KR) * TB, vslot = (u % VR) * TB;
        f32x16 s_nxt;
#pragma unroll
        for (int v = 0; v < 16; ++v) s_nxt[v] = 0.f;
        if (u + 1 <= last_w) {
#pragma unroll
          for (int kk = 0; kk < 8; ++kk)
            s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kread(kslot_n, kk), qreg[kk], s_nxt, 0, 0, 0);
        }
        const int k0 = u * UK;
        bf16x8 pb[2];
        softmax(s_cur, pb, (CAUSAL && k0 + UK - 1 > wq0) || (k0 + UK > n), k0);
#pragma unroll
        for (int sl = 0; sl < 2; ++sl)
#pragma unroll
          for (int db = 0; db < 4; ++db)
            oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vread(vslot, sl, db), pb[sl], oacc[db], 0, 0, 0);
        s_cur = s_nxt;
      }
      if (u <= u_sync_last) {
        __builtin_amdgcn_s_waitcnt(kVmcnt0);
        __syncthreads();
      }
    }
    __syncthreads();

    // ---- epilogue: O^T -> row-major through LDS (all units are dead: every wavefront passed the barrier above)
    char *Os = smem + wave * (WQ * OS_STRIDE * 2);
    {
      const float l = both_sum(lsum);
      const float inv = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int d0 = 32 * db + 8 * q4 + 4 * hh;
          u32x2 w = {pack_bf16(oacc[db][4 * q4] * inv, oacc[db][4 * q4 + 1] * inv),
                     pack_bf16(oacc[db][4 * q4 + 2] * inv, oacc[db][4 * q4 + 3] * inv)};
          *(u32x2 *)(Os + (ql * OS_STRIDE + d0) * 2) = w;
        }
    }
    __syncthreads();
    for (int p = lane; p < WQ * (D / 8); p += 64) {
      const int row = p / (D / 8), pc = p % (D / 8);
      if (wq0 + row < n)
        *(u32x4 *)(O + (t0 + wq0 + row) * q_stride + (int64_t)h * D + pc * 8) =
            *(const u32x4 *)(Os + (row * OS_STRIDE + pc * 8) * 2);
    }
  }
}

// ------------------------------------------------------------------------------------------ f32
// 64 queries per workgroup, four lanes per query (each owns D/4 channels), 32-key tiles in LDS.
template <int D, bool CAUSAL>
__global__ void __launch_bounds__(kThreads)
prefill_f32_kernel(const float *__restrict__ Q, const float *__restrict__ K, const float *__restrict__ V,
                   float *__restrict__ O, const int32_t *__restrict__ cu_seqlens, int Hq, int Hkv, int total_tokens,
                   int max_seqlen, float scale) {
  constexpr int QB = 64, KB = 32, C = D / 4;
  __shared__ float Ks[KB][D + 4];
  __shared__ float Vs[KB][D + 4];
  const int s = blockIdx.z, h = blockIdx.y, q0 = blockIdx.x * QB;
  int t0, n;
  seq_range(cu_seqlens, s, total_tokens, max_seqlen, t0, n);
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

hipError_t launch_bf16_d128(const lkv_ctx *c, const void *Q, const void *K, const void *V, void *O, const int32_t *cu,
                            int num_seqs, int max_seqlen, int64_t total_tokens, int causal, hipStream_t s) {
  constexpr int D = 128, BMQ = 128;
  // the kernel addresses a sequence's K/V rows with 32-bit byte offsets
  if ((int64_t)max_seqlen * c->cfg.num_kv_heads * D * 2 >= ((int64_t)1 << 32)) return hipErrorInvalidValue;
  const int Hq = c->cfg.num_q_heads, Hkv = c->cfg.num_kv_heads;
  const int tiles = (max_seqlen + BMQ - 1) / BMQ, halves = (tiles + 1) / 2;
  // Work slots per head: the sum over the sequences of ceil(n / 256) is at most (T + 255 * num_seqs) / 256, and never
  // more than every sequence being as long as the longest.
  int64_t slots = (total_tokens + (int64_t)255 * num_seqs) / 256;
  if (slots > (int64_t)halves * num_seqs) slots = (int64_t)halves * num_seqs;
  const int64_t grid_wgs = slots * Hq;
  if (grid_wgs > INT32_MAX) return hipErrorInvalidValue;
  const int xcd_heads = Hkv % kXcds == 0;
  const float sl2 = c->scale * kLog2e;
  dim3 grid((unsigned)grid_wgs);
  if (causal)
    launch_timed(c, true, true, prefill_bf16_d128_kernel<true>, grid, dim3(kThreads), s, (const uint16_t *)Q,
                       (const uint16_t *)K, (const uint16_t *)V, (uint16_t *)O, cu, Hq, Hkv, num_seqs, xcd_heads, (int)total_tokens,
                       max_seqlen, sl2);
  else
    launch_timed(c, true, true, prefill_bf16_d128_kernel<false>, grid, dim3(kThreads), s, (const uint16_t *)Q,
                       (const uint16_t *)K, (const uint16_t *)V, (uint16_t *)O, cu, Hq, Hkv, num_seqs, xcd_heads, (int)total_tokens,
                       max_seqlen, sl2);
  return hipGetLastError();
}

template <int D>
hipError_t launch_bf16(const lkv_ctx *c, const void *Q, const void *K, const void *V, void *O, const int32_t *cu,
                       int num_seqs, int max_seqlen, int64_t total_tokens, int causal, hipStream_t s) {
  constexpr int QB = 1, BMQ = 128 * QB;
  // the kernel addresses a sequence's K/V rows with 32-bit byte offsets
  if ((int64_t)max_seqlen * c->cfg.num_kv_heads * D * 2 >= ((int64_t)1 << 32)) return hipErrorInvalidValue;
  const int tiles = (max_seqlen + BMQ - 1) / BMQ;
  const int64_t total = (int64_t)c->cfg.num_q_heads * num_seqs * tiles;
  if (total > INT32_MAX) return hipErrorInvalidValue;
  const float sl2 = c->scale * kLog2e;
  dim3 grid((unsigned)total);
  if (causal)
    launch_timed(c, true, true, prefill_bf16_kernel<D, true, QB>, grid, dim3(kThreads), s, (const uint16_t *)Q,
                       (const uint16_t *)K, (const uint16_t *)V, (uint16_t *)O, cu, c->cfg.num_q_heads,
                       c->cfg.num_kv_heads, tiles, (int)total, (int)total_tokens, max_seqlen, sl2);
  else
    launch_timed(c, true, true, prefill_bf16_kernel<D, false, QB>, grid, dim3(kThreads), s, (const uint16_t *)Q,
                       (const uint16_t *)K, (const uint16_t *)V, (uint16_t *)O, cu, c->cfg.num_q_heads,
                       c->cfg.num_kv_heads, tiles, (int)total, (int)total_tokens, max_seqlen, sl2);
  return hipGetLastError();
}

template <int D>
hipError_t launch_f32(const lkv_ctx *c, const void *Q, const void *K, const void *V, void *O, const int32_t *cu,
                      int num_seqs, int max_seqlen, int64_t total_tokens, int causal, hipStream_t s) {
  dim3 grid((unsigned)((max_seqlen + 63) / 64), (unsigned)c->cfg.num_q_heads, (unsigned)num_seqs);
  if (causal)
    launch_timed(c, true, true, prefill_f32_kernel<D, true>, grid, dim3(kThreads), s, (const float *)Q, (const float *)K,
                       (const float *)V, (float *)O, cu, c->cfg.num_q_heads, c->cfg.num_kv_heads, (int)total_tokens, max_seqlen,
                       c->scale);
  else
    launch_timed(c, true, true, prefill_f32_kernel<D, false>, grid, dim3(kThreads), s, (const float *)Q, (const float *)K,
                       (const float *)V, (float *)O, cu, c->cfg.num_q_heads, c->cfg.num_kv_heads, (int)total_tokens, max_seqlen,
                       c->scale);
  return hipGetLastError();
}

}  // namespace

namespace lkv {

bool prefill_supported(const lkv_ctx *c) { return c->cfg.head_dim == 64 || c->cfg.head_dim == 128; }

hipError_t launch_prefill(const lkv_ctx *c, const void *Q, const void *K, const void *V, void *O, const int32_t *cu,
                          int32_t num_seqs, int32_t max_seqlen, int64_t total_tokens, int32_t causal, hipStream_t s) {
  // token offsets are 32-bit in cu_seqlens and in the kernels
  if (c->cfg.num_q_heads > 65535 || num_seqs > 65535 || total_tokens > INT32_MAX) return hipErrorInvalidValue;
  if (c->cfg.dtype == LKV_F32)
    return c->cfg.head_dim == 64 ? launch_f32<64>(c, Q, K, V, O, cu, num_seqs, max_seqlen, total_tokens, causal, s)
                                 : launch_f32<128>(c, Q, K, V, O, cu, num_seqs, max_seqlen, total_tokens, causal, s);
  return c->cfg.head_dim == 64 ? launch_bf16<64>(c, Q, K, V, O, cu, num_seqs, max_seqlen, total_tokens, causal, s)
                               : launch_bf16_d128(c, Q, K, V, O, cu, num_seqs, max_seqlen, total_tokens, causal, s);
}

}  // namespace lkv
