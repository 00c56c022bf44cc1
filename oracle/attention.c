/*
 * CPU oracle for the attention steps of the layer-wise paged KV cache -- TEST INFRASTRUCTURE.
 *
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may call this.  It
 * shares no code with the HIP library and is written straight from the definitions:
 *
 *   - softmax attention, causal in the prefill phase (paper Section 2.1.1: every prompt
 *     token is processed in parallel and attends to the tokens before it; cost quadratic
 *     in the prompt length);
 *   - attention of one new token over keys/values that live in non-contiguous blocks
 *     reached through a block table (paper Sections 2.1.2 and 2.2: the PagedAttention
 *     kernel used for decoding iterations), where every layer of a request has its own
 *     table (Section 3.2.2: block locations differ between layers).
 *
 * For one query row q, keys k_0..k_{n-1} and values v_0..v_{n-1}:
 *     s_j = scale * <q, k_j>;   m = max_j s_j;   p_j = exp(s_j - m);
 *     o   = (sum_j p_j v_j) / (sum_j p_j),
 * taken in ascending j with no blocking or reordering.  Accumulators are ACC_T (double in
 * the build used for parity, float in the build used to bound fp32 rounding).  Inputs are
 * float32 or bfloat16 bit patterns (widened exactly); outputs are written as double.
 *
 * Layout of a layer-block in the pool (the documented storage format, see lkv.h):
 *     [num_kv_heads][2: K then V][block_size][head_dim], block b at element offset
 *     b * num_kv_heads * 2 * block_size * head_dim.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef ACC_T
#define ACC_T double
#endif
#ifndef SUFFIX
#define SUFFIX f64
#endif
#define CAT2(a, b) a##_##b
#define CAT(a, b) CAT2(a, b)
#define FN(name) CAT(name, SUFFIX)

enum { DT_F32 = 0, DT_BF16 = 1 };

static inline float load_elem(const void *base, int64_t idx, int dtype) {
    if (dtype == DT_F32) return ((const float *)base)[idx];
    uint32_t u = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* Where row j of K and of V live: either a dense token-major tensor or the paged pool. */
typedef struct {
    int paged;
    /* dense: element offset of (token 0 of this sequence, this kv head); row stride in elements */
    const void *k, *v;
    int64_t base, stride;
    /* paged */
    const void *pool;
    const int32_t *table; /* this sequence's block ids for this layer */
    int64_t block_elems;  /* Hkv*2*bs*d */
    int64_t head_off;     /* g*2*bs*d */
    int bs, d;
} kv_src;

static inline void kv_row(const kv_src *s, int64_t j, const void **kb, int64_t *ko, const void **vb, int64_t *vo) {
    if (!s->paged) {
        *kb = s->k; *vb = s->v;
        *ko = *vo = s->base + j * s->stride;
    } else {
        int64_t blk = s->table[j / s->bs];
        int64_t off = blk * s->block_elems + s->head_off + (j % s->bs) * (int64_t)s->d;
        *kb = *vb = s->pool;
        *ko = off;
        *vo = off + (int64_t)s->bs * s->d;
    }
}

/* One query row against keys/values 0..n-1.  q points at d elements (index qo). */
static void attend_row(const void *q, int64_t qo, int dtype, const kv_src *src, int64_t n, int d,
                       double scale, double *out, ACC_T *scratch /* n */) {
    if (n <= 0) { /* nothing to attend to: defined as a zero row */
        for (int c = 0; c < d; ++c) out[c] = 0.0;
        return;
    }
    ACC_T m = -INFINITY;
    for (int64_t j = 0; j < n; ++j) {
        const void *kb, *vb; int64_t ko, vo;
        kv_row(src, j, &kb, &ko, &vb, &vo);
        ACC_T dot = 0;
        for (int c = 0; c < d; ++c)
            dot += (ACC_T)load_elem(q, qo + c, dtype) * (ACC_T)load_elem(kb, ko + c, dtype);
        ACC_T s = (ACC_T)scale * dot;
        scratch[j] = s;
        if (s > m) m = s;
    }
    ACC_T denom = 0;
    ACC_T acc[512];
    for (int c = 0; c < d; ++c) acc[c] = 0;
    for (int64_t j = 0; j < n; ++j) {
        const void *kb, *vb; int64_t ko, vo;
        kv_row(src, j, &kb, &ko, &vb, &vo);
        ACC_T p = (sizeof(ACC_T) == sizeof(double)) ? (ACC_T)exp((double)(scratch[j] - m))
                                                    : (ACC_T)expf((float)(scratch[j] - m));
        denom += p;
        for (int c = 0; c < d; ++c) acc[c] += p * (ACC_T)load_elem(vb, vo + c, dtype);
    }
    for (int c = 0; c < d; ++c) out[c] = (double)(acc[c] / denom);
}

/*
 * Prefill attention on packed variable-length sequences.
 * Q [T][Hq][d], K,V [T][Hkv][d]; cu_seqlens [B+1]; O [T][Hq][d] (double).
 * Row i of a sequence sees keys 0..i when causal, 0..n-1 otherwise.
 * q head h uses kv head h / (Hq/Hkv).  Returns 0, or -1 on bad arguments.
 */
int FN(orc_prefill_attention)(const void *Q, const void *K, const void *V, double *O,
                              const int32_t *cu_seqlens, int num_seqs, int Hq, int Hkv, int d,
                              double scale, int causal, int dtype, int nthreads) {
    if (Hq <= 0 || Hkv <= 0 || Hq % Hkv || d <= 0 || d > 512) return -1;
    int group = Hq / Hkv;
    int64_t maxn = 0;
    for (int s = 0; s < num_seqs; ++s) {
        int64_t n = cu_seqlens[s + 1] - cu_seqlens[s];
        if (n > maxn) maxn = n;
    }
    (void)nthreads;
#pragma omp parallel num_threads(nthreads > 0 ? nthreads : 1)
    {
        ACC_T *scratch = (ACC_T *)malloc(sizeof(ACC_T) * (size_t)(maxn > 0 ? maxn : 1));
#pragma omp for collapse(2) schedule(dynamic, 1)
        for (int s = 0; s < num_seqs; ++s) {
            for (int h = 0; h < Hq; ++h) {
                int64_t t0 = cu_seqlens[s], n = cu_seqlens[s + 1] - cu_seqlens[s];
                kv_src src;
                memset(&src, 0, sizeof src);
                src.paged = 0; src.k = K; src.v = V;
                src.base = (t0 * Hkv + h / group) * (int64_t)d;
                src.stride = (int64_t)Hkv * d;
                for (int64_t i = 0; i < n; ++i) {
                    int64_t qo = ((t0 + i) * Hq + h) * (int64_t)d;
                    attend_row(Q, qo, dtype, &src, causal ? i + 1 : n, d, scale, O + qo, scratch);
                }
            }
        }
        free(scratch);
    }
    return 0;
}

/*
 * The same, for a list of sampled (token, head) output rows only (for sizes where the full
 * result is out of reach).  tok[i] is a global token index into the packed tensors.
 * O_rows [n_rows][d].
 */
int FN(orc_prefill_attention_rows)(const void *Q, const void *K, const void *V, double *O_rows,
                                   const int32_t *cu_seqlens, int num_seqs, int Hq, int Hkv, int d,
                                   double scale, int causal, int dtype,
                                   const int64_t *tok, const int32_t *head, int64_t n_rows, int nthreads) {
    if (Hq <= 0 || Hkv <= 0 || Hq % Hkv || d <= 0 || d > 512) return -1;
    int group = Hq / Hkv;
    int bad = 0;
    (void)nthreads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
    for (int64_t r = 0; r < n_rows; ++r) {
        int s = -1;
        for (int c = 0; c < num_seqs; ++c)
            if (tok[r] >= cu_seqlens[c] && tok[r] < cu_seqlens[c + 1]) s = c;
        if (s < 0 || head[r] < 0 || head[r] >= Hq) { bad = 1; continue; }
        int64_t t0 = cu_seqlens[s], n = cu_seqlens[s + 1] - t0, i = tok[r] - t0;
        int64_t nk = causal ? i + 1 : n;
        ACC_T *scratch = (ACC_T *)malloc(sizeof(ACC_T) * (size_t)nk);
        kv_src src;
        memset(&src, 0, sizeof src);
        src.paged = 0; src.k = K; src.v = V;
        src.base = (t0 * Hkv + head[r] / group) * (int64_t)d;
        src.stride = (int64_t)Hkv * d;
        attend_row(Q, (tok[r] * Hq + head[r]) * (int64_t)d, dtype, &src, nk, d, scale, O_rows + r * d, scratch);
        free(scratch);
    }
    return bad ? -1 : 0;
}

/*
 * Decode attention through a block table.
 * Q [B][Hq][d]; pool = all layer-blocks; block_table [B][max_blocks] (this layer's ids,
 * unused entries ignored); context_lens [B]; O [B][Hq][d] (double).
 * Sequence s attends to positions 0..context_lens[s]-1; a zero context gives a zero row.
 */
int FN(orc_paged_decode_attention)(const void *Q, const void *pool, double *O,
                                   const int32_t *block_table, int max_blocks,
                                   const int32_t *context_lens, int num_seqs,
                                   int Hq, int Hkv, int d, int bs, int64_t num_pool_blocks,
                                   double scale, int dtype, int nthreads) {
    if (Hq <= 0 || Hkv <= 0 || Hq % Hkv || d <= 0 || d > 512 || bs <= 0) return -1;
    int group = Hq / Hkv;
    int64_t maxn = 1;
    for (int s = 0; s < num_seqs; ++s) {
        int64_t n = context_lens[s];
        if (n < 0 || (n + bs - 1) / bs > max_blocks) return -1;
        for (int64_t b = 0; b < (n + bs - 1) / bs; ++b) {
            int32_t id = block_table[(int64_t)s * max_blocks + b];
            if (id < 0 || id >= num_pool_blocks) return -1;
        }
        if (n > maxn) maxn = n;
    }
    (void)nthreads;
#pragma omp parallel num_threads(nthreads > 0 ? nthreads : 1)
    {
        ACC_T *scratch = (ACC_T *)malloc(sizeof(ACC_T) * (size_t)maxn);
#pragma omp for collapse(2) schedule(dynamic, 1)
        for (int s = 0; s < num_seqs; ++s) {
            for (int h = 0; h < Hq; ++h) {
                kv_src src;
                memset(&src, 0, sizeof src);
                src.paged = 1; src.pool = pool;
                src.table = block_table + (int64_t)s * max_blocks;
                src.block_elems = (int64_t)Hkv * 2 * bs * d;
                src.head_off = (int64_t)(h / group) * 2 * bs * d;
                src.bs = bs; src.d = d;
                int64_t qo = ((int64_t)s * Hq + h) * d;
                attend_row(Q, qo, dtype, &src, context_lens[s], d, scale, O + qo, scratch);
            }
        }
        free(scratch);
    }
    return 0;
}
