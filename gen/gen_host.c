/*
 * Seeded synthetic-input generator (host side).
 *
 * This module only manufactures test inputs: counter-based random numbers
 * (Philox4x32-10 keyed through FNV-1a-64), Box-Muller normals and row-wise
 * log_softmax.  It holds none of the decoding method's arithmetic and is the
 * only code that the CPU oracle's tests and the GPU library's tests share.
 *
 * Recipe (all arithmetic fp64, results rounded to fp32 once at the end):
 *   key64   = FNV-1a-64 over the little-endian bytes of
 *             (seed:u64, tag:u32, a:u32, b:u32, c:u64)
 *   Philox  key = (lo32(key64), hi32(key64)), counter = (block, 0, 0, 0)
 *   block i yields r0..r3; u = (r + 0.5) / 2^32;
 *             z[4i+0] = sqrt(-2 ln u0) cos(2 pi u1), z[4i+1] = ... sin(...)
 *             z[4i+2], z[4i+3] likewise from (u2, u3)
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define GEN_TAG_CTC_LOGIT 1u
#define GEN_TAG_CTC_BOOST 2u
#define GEN_TAG_ATT       3u
#define GEN_TAG_LENGTH    4u
#define GEN_TAG_MISC      5u

uint64_t gen_fnv1a64(const void* data, size_t n, uint64_t h) {
  const unsigned char* p = (const unsigned char*)data;
  for (size_t i = 0; i < n; ++i) {
    h ^= (uint64_t)p[i];
    h *= 0x100000001b3ull;
  }
  return h;
}

uint64_t gen_fnv_basis(void) { return 0xcbf29ce484222325ull; }

/* Hash of a label sequence: FNV-1a-64 over the little-endian int32 labels. */
uint64_t gen_prefix_hash(const int32_t* labels, int n) {
  uint64_t h = gen_fnv_basis();
  for (int i = 0; i < n; ++i) {
    uint32_t v = (uint32_t)labels[i];
    unsigned char b[4] = {(unsigned char)(v), (unsigned char)(v >> 8),
                          (unsigned char)(v >> 16), (unsigned char)(v >> 24)};
    h = gen_fnv1a64(b, 4, h);
  }
  return h;
}

uint64_t gen_prefix_hash_extend(uint64_t h, int32_t label) {
  uint32_t v = (uint32_t)label;
  unsigned char b[4] = {(unsigned char)(v), (unsigned char)(v >> 8),
                        (unsigned char)(v >> 16), (unsigned char)(v >> 24)};
  return gen_fnv1a64(b, 4, h);
}

static void put32(unsigned char* p, uint32_t v) {
  p[0] = (unsigned char)v; p[1] = (unsigned char)(v >> 8);
  p[2] = (unsigned char)(v >> 16); p[3] = (unsigned char)(v >> 24);
}

uint64_t gen_stream_key(uint64_t seed, uint32_t tag, uint32_t a, uint32_t b, uint64_t c) {
  unsigned char buf[28];
  put32(buf, (uint32_t)seed); put32(buf + 4, (uint32_t)(seed >> 32));
  put32(buf + 8, tag); put32(buf + 12, a); put32(buf + 16, b);
  put32(buf + 20, (uint32_t)c); put32(buf + 24, (uint32_t)(c >> 32));
  return gen_fnv1a64(buf, sizeof buf, gen_fnv_basis());
}

void gen_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int r = 0; r < 10; ++r) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

static void block_normals(uint64_t key64, uint32_t block, double z[4]) {
  uint32_t ctr[4] = {block, 0u, 0u, 0u};
  uint32_t key[2] = {(uint32_t)key64, (uint32_t)(key64 >> 32)};
  uint32_t r[4];
  gen_philox4x32_10(ctr, key, r);
  const double inv = 1.0 / 4294967296.0;
  const double two_pi = 6.283185307179586476925286766559;
  for (int h = 0; h < 2; ++h) {
    double u0 = ((double)r[2 * h] + 0.5) * inv;
    double u1 = ((double)r[2 * h + 1] + 0.5) * inv;
    double rad = sqrt(-2.0 * log(u0));
    z[2 * h] = rad * cos(two_pi * u1);
    z[2 * h + 1] = rad * sin(two_pi * u1);
  }
}

/* n standard normals of the stream `key64`, element e = lane e%4 of block e/4. */
void gen_normals(uint64_t key64, size_t n, double* out) {
  for (size_t b = 0; b * 4 < n; ++b) {
    double z[4];
    block_normals(key64, (uint32_t)b, z);
    for (int j = 0; j < 4 && b * 4 + j < n; ++j) out[b * 4 + j] = z[j];
  }
}

/* n uniforms in (0,1) of the stream `key64` (one 32-bit draw each). */
void gen_uniforms(uint64_t key64, size_t n, double* out) {
  const double inv = 1.0 / 4294967296.0;
  for (size_t b = 0; b * 4 < n; ++b) {
    uint32_t ctr[4] = {(uint32_t)b, 0u, 0u, 0u};
    uint32_t key[2] = {(uint32_t)key64, (uint32_t)(key64 >> 32)};
    uint32_t r[4];
    gen_philox4x32_10(ctr, key, r);
    for (int j = 0; j < 4 && b * 4 + j < n; ++j) out[b * 4 + j] = ((double)r[j] + 0.5) * inv;
  }
}

static void log_softmax_row(const double* logit, int n, float* out) {
  double m = logit[0];
  for (int i = 1; i < n; ++i) if (logit[i] > m) m = logit[i];
  double s = 0.0;
  for (int i = 0; i < n; ++i) s += exp(logit[i] - m);
  double lse = m + log(s);
  for (int i = 0; i < n; ++i) out[i] = (float)(logit[i] - lse);
}

/*
 * Utterance lengths: T_i uniform on the integers lo..hi.
 */
void gen_lengths(uint64_t seed, int n_utt, int lo, int hi, int32_t* out) {
  uint64_t key = gen_stream_key(seed, GEN_TAG_LENGTH, 0u, 0u, 0ull);
  double* u = (double*)malloc(sizeof(double) * (size_t)(n_utt > 0 ? n_utt : 1));
  gen_uniforms(key, (size_t)n_utt, u);
  for (int i = 0; i < n_utt; ++i) {
    int span = hi - lo + 1;
    int v = lo + (int)(u[i] * span);
    if (v > hi) v = hi;
    out[i] = v;
  }
  free(u);
}

/*
 * Blank-peaky CTC log-posteriors of one utterance, out[t*V + k], t = 0..T-1
 * (frame t+1 of the paper's 1-based numbering).
 *   logit[k] = N(0,1); non-blank k gets + log(rank^-zipf_s / Z) with rank = its
 *   position among the non-blank ids (zipf_s = 0: no prior); the blank id gets
 *   + blank_boost on frames drawn Bernoulli(p_boost); row log_softmax.
 */
void gen_ctc_utt(uint64_t seed, uint32_t utt, int T, int V, int blank_id,
                 double blank_boost, double p_boost, double zipf_s, float* out) {
  double* prior = (double*)calloc((size_t)V, sizeof(double));
  if (zipf_s > 0.0) {
    double Z = 0.0;
    for (int r = 1; r <= V - 1; ++r) Z += pow((double)r, -zipf_s);
    int r = 1;
    for (int k = 0; k < V; ++k) {
      if (k == blank_id) continue;
      prior[k] = -zipf_s * log((double)r) - log(Z);
      ++r;
    }
  }
  double* boost_u = (double*)malloc(sizeof(double) * (size_t)T);
  gen_uniforms(gen_stream_key(seed, GEN_TAG_CTC_BOOST, utt, 0u, 0ull), (size_t)T, boost_u);
  double* logit = (double*)malloc(sizeof(double) * (size_t)V);
  for (int t = 0; t < T; ++t) {
    gen_normals(gen_stream_key(seed, GEN_TAG_CTC_LOGIT, utt, (uint32_t)t, 0ull), (size_t)V, logit);
    for (int k = 0; k < V; ++k) logit[k] += prior[k];
    if (boost_u[t] < p_boost) logit[blank_id] += blank_boost;
    log_softmax_row(logit, V, out + (size_t)t * V);
  }
  free(logit); free(boost_u); free(prior);
}

/*
 * One attention log-probability row: log_softmax(scale * N(0,1)) over V ids,
 * the stream keyed by (seed, utt, step, hash of the hypothesis's labels).
 */
void gen_att_row(uint64_t seed, uint32_t utt, uint32_t step, uint64_t prefix_hash,
                 int V, double scale, float* out) {
  double* logit = (double*)malloc(sizeof(double) * (size_t)V);
  gen_normals(gen_stream_key(seed, GEN_TAG_ATT, utt, step, prefix_hash), (size_t)V, logit);
  for (int k = 0; k < V; ++k) logit[k] *= scale;
  log_softmax_row(logit, V, out);
  free(logit);
}

/* Rows for several hypotheses of several utterances at once (parallel over rows). */
void gen_att_rows(uint64_t seed, const uint32_t* utt, uint32_t step, const uint64_t* prefix_hash,
                  int n_rows, int V, double scale, float* out) {
#pragma omp parallel for schedule(dynamic)
  for (int r = 0; r < n_rows; ++r)
    gen_att_row(seed, utt[r], step, prefix_hash[r], V, scale, out + (size_t)r * V);
}

void gen_ctc_batch(uint64_t seed, int n_utt, const int32_t* lens, int t_max, int V, int blank_id,
                   double blank_boost, double p_boost, double zipf_s, float pad_value, float* out) {
#pragma omp parallel for schedule(dynamic)
  for (int u = 0; u < n_utt; ++u) {
    float* base = out + (size_t)u * t_max * V;
    gen_ctc_utt(seed, (uint32_t)u, lens[u], V, blank_id, blank_boost, p_boost, zipf_s, base);
    for (size_t i = (size_t)lens[u] * V; i < (size_t)t_max * V; ++i) base[i] = pad_value;
  }
}
