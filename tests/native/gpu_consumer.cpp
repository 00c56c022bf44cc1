// A consumer of the C ABI that is not Python and owns no torch memory: plain HIP runtime calls for the buffers,
// the library for everything else.  One bf16 layer of two prompts goes through write, causal prefill attention,
// offload to pinned memory, release, reload into other blocks and decode; the results are checked against a dense
// double-precision attention written out here (Section 2.1.1) and against each other.  Exit code 0 = all held.
//
//   hipcc -std=c++17 -I include tests/native/gpu_consumer.cpp -L paper_2410_00428_amd -llkv -o gpu_consumer
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "lkv.h"

#define HIP(x)                                                                                   \
  do {                                                                                           \
    hipError_t e_ = (x);                                                                         \
    if (e_ != hipSuccess) {                                                                      \
      std::fprintf(stderr, "gpu_consumer: %s: %s (line %d)\n", #x, hipGetErrorString(e_), __LINE__); \
      return 2;                                                                                  \
    }                                                                                            \
  } while (0)
#define LKV(x)                                                                                            \
  do {                                                                                                    \
    lkv_status s_ = (x);                                                                                  \
    if (s_ != LKV_OK) {                                                                                   \
      std::fprintf(stderr, "gpu_consumer: %s -> %d: %s (line %d)\n", #x, (int)s_, lkv_last_error(c), __LINE__); \
      return 3;                                                                                           \
    }                                                                                                     \
  } while (0)
#define CHECK(x)                                                                    \
  do {                                                                              \
    if (!(x)) {                                                                     \
      std::fprintf(stderr, "gpu_consumer: %s does not hold (line %d)\n", #x, __LINE__); \
      return 1;                                                                     \
    }                                                                               \
  } while (0)

namespace {

uint16_t to_bf16(float f) {  // round to nearest, ties to even (finite inputs only)
  uint32_t u;
  std::memcpy(&u, &f, 4);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
float from_bf16(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

struct Lcg {  // small deterministic generator: sums of four uniforms, roughly bell-shaped around 0
  uint64_t s;
  float next() {
    float a = 0.f;
    for (int i = 0; i < 4; ++i) {
      s = s * 6364136223846793005ull + 1442695040888963407ull;
      a += (float)((s >> 40) & 0xFFFF) / 65536.f - 0.5f;
    }
    return a;
  }
};

// Row `i` of sequence [t0, t0+n) attends to keys t0..t0+last; head h uses kv head h / (Hq / Hkv).
void dense_row(const std::vector<uint16_t> &Q, const std::vector<uint16_t> &K, const std::vector<uint16_t> &V, int Hq,
               int Hkv, int d, int64_t qrow, int h, int64_t t0, int64_t last, double *out) {
  const int g = h / (Hq / Hkv);
  const double scale = 1.0 / std::sqrt((double)d);
  std::vector<double> s(last + 1);
  double m = -1e300;
  for (int64_t j = 0; j <= last; ++j) {
    double acc = 0;
    for (int e = 0; e < d; ++e)
      acc += (double)from_bf16(Q[(qrow * Hq + h) * d + e]) * (double)from_bf16(K[((t0 + j) * Hkv + g) * d + e]);
    s[j] = acc * scale;
    m = s[j] > m ? s[j] : m;
  }
  double l = 0;
  for (int e = 0; e < d; ++e) out[e] = 0;
  for (int64_t j = 0; j <= last; ++j) {
    const double p = std::exp(s[j] - m);
    l += p;
    for (int e = 0; e < d; ++e) out[e] += p * (double)from_bf16(V[((t0 + j) * Hkv + g) * d + e]);
  }
  for (int e = 0; e < d; ++e) out[e] /= l;
}

bool close_enough(const uint16_t *got, const double *ref, int d, double *worst) {
  bool ok = true;
  for (int e = 0; e < d; ++e) {
    const double err = std::fabs((double)from_bf16(got[e]) - ref[e]);
    if (err > *worst) *worst = err;
    if (!(err <= 2e-2 + 1e-2 * std::fabs(ref[e]))) ok = false;  // the bf16 bound of the parity tests
  }
  return ok;
}

}  // namespace

int main() {
  const int Hq = 4, Hkv = 2, d = 128, bs = 16;
  const int64_t lens[2] = {150, 37};  // two 128-query tiles with a ragged tail, and a short prompt
  const int64_t T = lens[0] + lens[1];
  const int32_t cu_host[3] = {0, (int32_t)lens[0], (int32_t)T};
  int ndev = 0;
  HIP(hipGetDeviceCount(&ndev));
  CHECK(ndev >= 1);
  HIP(hipSetDevice(0));

  lkv_ctx *c = nullptr;
  lkv_config cfg;
  std::memset(&cfg, 0, sizeof cfg);
  cfg.num_layers = 1;
  cfg.num_q_heads = Hq;
  cfg.num_kv_heads = Hkv;
  cfg.head_dim = d;
  cfg.block_size = bs;
  cfg.dtype = LKV_BF16;
  cfg.num_pool_blocks = 40;
  cfg.staging_bytes = 1 << 20;
  LKV(lkv_create(&cfg, &c));
  int32_t order[40];
  for (int i = 0; i < 40; ++i) order[i] = (i * 17 + 5) % 40;  // a permutation: 17 and 40 are coprime
  LKV(lkv_pool_reset(c, order, 40));

  Lcg rng{20241000428ull};
  std::vector<uint16_t> Q((size_t)T * Hq * d), K((size_t)T * Hkv * d), V((size_t)T * Hkv * d);
  for (auto &x : Q) x = to_bf16(rng.next());
  for (auto &x : K) x = to_bf16(rng.next());
  for (auto &x : V) x = to_bf16(rng.next());

  void *dQ, *dK, *dV, *dO, *dcu, *dslots, *dtable, *dctx, *dq1, *dO1, *dO2;
  HIP(hipMalloc(&dQ, Q.size() * 2));
  HIP(hipMalloc(&dK, K.size() * 2));
  HIP(hipMalloc(&dV, V.size() * 2));
  HIP(hipMalloc(&dO, Q.size() * 2));
  HIP(hipMalloc(&dcu, sizeof cu_host));
  HIP(hipMalloc(&dslots, T * 8));
  HIP(hipMalloc(&dq1, 2 * Hq * d * 2));
  HIP(hipMalloc(&dO1, 2 * Hq * d * 2));
  HIP(hipMalloc(&dO2, 2 * Hq * d * 2));
  HIP(hipMalloc(&dctx, 2 * 4));
  HIP(hipMemcpy(dQ, Q.data(), Q.size() * 2, hipMemcpyHostToDevice));
  HIP(hipMemcpy(dK, K.data(), K.size() * 2, hipMemcpyHostToDevice));
  HIP(hipMemcpy(dV, V.data(), V.size() * 2, hipMemcpyHostToDevice));
  HIP(hipMemcpy(dcu, cu_host, sizeof cu_host, hipMemcpyHostToDevice));
  hipStream_t main_s, side_s;
  HIP(hipStreamCreate(&main_s));
  HIP(hipStreamCreate(&side_s));

  // allocate + map, write, prefill
  std::vector<int64_t> slots(T);
  for (int s = 0; s < 2; ++s) {
    LKV(lkv_alloc_layer_blocks(c, s, 0, lens[s]));
    LKV(lkv_build_slot_mapping(c, s, 0, 0, lens[s], slots.data() + cu_host[s]));
  }
  CHECK(lkv_num_free_blocks(c) == 40 - 10 - 3);
  HIP(hipMemcpy(dslots, slots.data(), T * 8, hipMemcpyHostToDevice));
  LKV(lkv_write_kv(c, 0, dK, dV, (const int64_t *)dslots, T, main_s));
  LKV(lkv_prefill_attention(c, 0, dQ, dK, dV, dO, (const int32_t *)dcu, 2, (int32_t)lens[0], T, 1, main_s));
  HIP(hipStreamSynchronize(main_s));
  std::vector<uint16_t> O(Q.size());
  HIP(hipMemcpy(O.data(), dO, O.size() * 2, hipMemcpyDeviceToHost));
  std::vector<double> ref(d);
  double worst = 0;
  const int64_t rows[] = {0, 15, 16, 127, 128, 149, 150, 151, 186};  // first / last rows of blocks, tiles, sequences
  for (int64_t r : rows)
    for (int h = 0; h < Hq; ++h) {
      const int s = r < lens[0] ? 0 : 1;
      dense_row(Q, K, V, Hq, Hkv, d, r, h, cu_host[s], r - cu_host[s], ref.data());
      CHECK(close_enough(&O[(r * Hq + h) * d], ref.data(), d, &worst));
    }

  // decode with the last query of each prompt over the whole context: the same numbers as its causal row
  int32_t table[2][10], ctx_host[2] = {(int32_t)lens[0], (int32_t)lens[1]};
  std::memset(table, 0xFF, sizeof table);
  std::vector<uint16_t> q1((size_t)2 * Hq * d);
  for (int s = 0; s < 2; ++s) {
    int64_t n = 0;
    LKV(lkv_get_block_table(c, s, 0, table[s], 10, &n));
    CHECK(n == (lens[s] + bs - 1) / bs);
    std::memcpy(&q1[(size_t)s * Hq * d], &Q[(size_t)(cu_host[s + 1] - 1) * Hq * d], (size_t)Hq * d * 2);
  }
  HIP(hipMalloc(&dtable, sizeof table));
  HIP(hipMemcpy(dtable, table, sizeof table, hipMemcpyHostToDevice));
  HIP(hipMemcpy(dctx, ctx_host, sizeof ctx_host, hipMemcpyHostToDevice));
  HIP(hipMemcpy(dq1, q1.data(), q1.size() * 2, hipMemcpyHostToDevice));
  LKV(lkv_paged_decode_attention(c, 0, dq1, dO1, (const int32_t *)dtable, 10, (const int32_t *)dctx, 2, main_s));
  HIP(hipStreamSynchronize(main_s));
  std::vector<uint16_t> O1(q1.size()), O2(q1.size());
  HIP(hipMemcpy(O1.data(), dO1, O1.size() * 2, hipMemcpyDeviceToHost));
  for (int s = 0; s < 2; ++s)
    for (int h = 0; h < Hq; ++h) {
      const int64_t r = cu_host[s + 1] - 1;
      dense_row(Q, K, V, Hq, Hkv, d, r, h, cu_host[s], lens[s] - 1, ref.data());
      CHECK(close_enough(&O1[((size_t)s * Hq + h) * d], ref.data(), d, &worst));
    }

  // offload on the side stream, release, reload into whatever blocks come next, decode again: the same bits
  int64_t block_bytes = 0;
  LKV(lkv_pool_info(c, nullptr, nullptr, &block_bytes));
  CHECK(block_bytes == 2 * Hkv * d * bs * 2);
  int32_t ids[13];
  std::memcpy(ids, table[0], 10 * 4);
  std::memcpy(ids + 10, table[1], 3 * 4);
  void *image;
  HIP(hipHostMalloc(&image, 13 * block_bytes, hipHostMallocDefault));
  LKV(lkv_pack_layer_blocks(c, 0, ids, 13, image, side_s));
  LKV(lkv_event_synchronize(c, 0, LKV_EV_OFFLOADED));
  for (int s = 0; s < 2; ++s) LKV(lkv_free_layer_blocks(c, s, 0, 1));
  CHECK(lkv_num_free_blocks(c) == 40);
  int32_t res = -1;
  LKV(lkv_layer_residency(c, 0, 0, &res));
  CHECK(res == LKV_RES_HOST);
  LKV(lkv_alloc_layer_blocks(c, 1, 0, lens[1]));  // the other order: the blocks differ from the first time
  LKV(lkv_alloc_layer_blocks(c, 0, 0, lens[0]));
  int32_t table2[2][10], ids2[13];
  std::memset(table2, 0xFF, sizeof table2);
  for (int s = 0; s < 2; ++s) {
    int64_t n = 0;
    LKV(lkv_get_block_table(c, s, 0, table2[s], 10, &n));
  }
  CHECK(std::memcmp(table, table2, sizeof table) != 0);
  std::memcpy(ids2, table2[0], 10 * 4);
  std::memcpy(ids2 + 10, table2[1], 3 * 4);
  LKV(lkv_unpack_layer_blocks(c, 0, ids2, 13, image, side_s));
  HIP(hipMemcpyAsync(dtable, table2, sizeof table2, hipMemcpyHostToDevice, main_s));
  LKV(lkv_paged_decode_attention(c, 0, dq1, dO2, (const int32_t *)dtable, 10, (const int32_t *)dctx, 2, main_s));  // waits for the reload
  HIP(hipStreamSynchronize(main_s));
  HIP(hipMemcpy(O2.data(), dO2, O2.size() * 2, hipMemcpyDeviceToHost));
  CHECK(std::memcmp(O1.data(), O2.data(), O1.size() * 2) == 0);

  lkv_stats st;
  LKV(lkv_get_stats(c, &st, (int64_t)sizeof st));
  CHECK(st.write_kv_calls == 1 && st.prefill_calls == 1 && st.decode_calls == 2 && st.pack_calls == 1 && st.unpack_calls == 1);
  CHECK(st.pack_bytes == 13 * block_bytes && st.unpack_bytes == 13 * block_bytes);
  lkv_destroy(c);
  HIP(hipHostFree(image));
  for (void *p : {dQ, dK, dV, dO, dcu, dslots, dtable, dctx, dq1, dO1, dO2}) HIP(hipFree(p));
  std::printf("gpu_consumer: ok (largest deviation from the dense double-precision attention %.2e)\n", worst);
  return 0;
}
