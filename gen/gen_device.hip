// Device twin of the synthetic-input generator (same recipe as gen_host.c, written straight
// into GPU memory for throughput runs).  Input manufacture only: none of the decoding
// method's arithmetic.  Its transcendental functions are the device's, so its bytes are not
// promised to equal the host generator's; whoever needs both sides to see the same input
// copies these bytes back.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#define TAG_CTC_LOGIT 1u
#define TAG_CTC_BOOST 2u
#define TAG_ATT 3u

__device__ __forceinline__ uint64_t fnv_bytes32(uint64_t h, uint32_t v) {
#pragma unroll
  for (int i = 0; i < 4; ++i) { h ^= (uint64_t)((v >> (8 * i)) & 0xffu); h *= 0x100000001b3ull; }
  return h;
}

__device__ __forceinline__ uint64_t stream_key(uint64_t seed, uint32_t tag, uint32_t a, uint32_t b, uint64_t c) {
  uint64_t h = 0xcbf29ce484222325ull;
  h = fnv_bytes32(h, (uint32_t)seed); h = fnv_bytes32(h, (uint32_t)(seed >> 32));
  h = fnv_bytes32(h, tag); h = fnv_bytes32(h, a); h = fnv_bytes32(h, b);
  h = fnv_bytes32(h, (uint32_t)c); h = fnv_bytes32(h, (uint32_t)(c >> 32));
  return h;
}

__device__ __forceinline__ void philox(uint32_t block, uint64_t key64, uint32_t r[4]) {
  uint32_t c0 = block, c1 = 0, c2 = 0, c3 = 0;
  uint32_t k0 = (uint32_t)key64, k1 = (uint32_t)(key64 >> 32);
#pragma unroll
  for (int i = 0; i < 10; ++i) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  r[0] = c0; r[1] = c1; r[2] = c2; r[3] = c3;
}

__device__ __forceinline__ void block_normals(uint64_t key, uint32_t block, double z[4]) {
  uint32_t r[4];
  philox(block, key, r);
  const double inv = 1.0 / 4294967296.0, two_pi = 6.283185307179586476925286766559;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    double u0 = ((double)r[2 * h] + 0.5) * inv, u1 = ((double)r[2 * h + 1] + 0.5) * inv;
    double rad = sqrt(-2.0 * log(u0));
    z[2 * h] = rad * cos(two_pi * u1);
    z[2 * h + 1] = rad * sin(two_pi * u1);
  }
}

__device__ __forceinline__ double block_reduce_max(double v, double* sh) {
  for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o));
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  double r = sh[0];
  for (int i = 1; i < (int)(blockDim.x >> 6); ++i) r = fmax(r, sh[i]);
  return r;
}
__device__ __forceinline__ double block_reduce_sum(double v, double* sh) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  double r = 0.0;
  for (int i = 0; i < (int)(blockDim.x >> 6); ++i) r += sh[i];
  return r;
}

// One row: logits[k] = scale * z[k] + prior(k) (+ boost on the blank id), then log_softmax.
// The row's logits are kept in dynamic LDS (V doubles).
__device__ void make_row(uint64_t key, int V, double scale, double zipf_s, double log_Z, int blank_id,
                         double blank_add, float* out, double* logit, double* sh) {
  const int tid = threadIdx.x;
  for (int b = tid; b * 4 < V; b += blockDim.x) {
    double z[4];
    block_normals(key, (uint32_t)b, z);
    for (int j = 0; j < 4; ++j) {
      int k = b * 4 + j;
      if (k >= V) break;
      double v = scale * z[j];
      if (zipf_s > 0.0 && k != blank_id) {
        int rank = k < blank_id ? k + 1 : k;          // position among the non-blank ids, 1-based
        v += -zipf_s * log((double)rank) - log_Z;
      }
      if (k == blank_id) v += blank_add;
      logit[k] = v;
    }
  }
  __syncthreads();
  double m = -INFINITY;
  for (int k = tid; k < V; k += blockDim.x) m = fmax(m, logit[k]);
  m = block_reduce_max(m, sh);
  double s = 0.0;
  for (int k = tid; k < V; k += blockDim.x) s += exp(logit[k] - m);
  s = block_reduce_sum(s, sh);
  const double lse = m + log(s);
  for (int k = tid; k < V; k += blockDim.x) out[k] = (float)(logit[k] - lse);
}

__global__ void k_gen_ctc(uint64_t seed, const int32_t* lens, int t_max, int V, int blank_id, double boost,
                          double p_boost, double zipf_s, double log_Z, float* out) {
  extern __shared__ double logit[];
  __shared__ double sh[16];
  const int t = blockIdx.x, u = blockIdx.y;
  if (t >= lens[u]) return;
  uint32_t r[4];
  philox((uint32_t)(t >> 2), stream_key(seed, TAG_CTC_BOOST, (uint32_t)u, 0u, 0ull), r);
  const double ub = ((double)r[t & 3] + 0.5) * (1.0 / 4294967296.0);
  const double add = ub < p_boost ? boost : 0.0;
  make_row(stream_key(seed, TAG_CTC_LOGIT, (uint32_t)u, (uint32_t)t, 0ull), V, 1.0, zipf_s, log_Z, blank_id,
           add, out + ((size_t)u * t_max + t) * V, logit, sh);
}

// Attention rows of one step.  Slot (u, n) holds the hypothesis that extends old slot
// parent[u][n] by token[u][n]; its prefix hash is the parent's hash extended by the token.
// first_step != 0: every utterance's slot 0 holds the empty hypothesis (hash = FNV basis).
__global__ void k_gen_att(uint64_t seed, uint32_t step, int Wb, int V, double scale, int first_step,
                          const uint64_t* hash_in, const int32_t* parent, const int32_t* token,
                          const uint8_t* live, uint64_t* hash_out, float* out) {
  extern __shared__ double logit[];
  __shared__ double sh[16];
  const int slot = blockIdx.x, u = slot / Wb, n = slot % Wb;
  uint64_t h;
  if (first_step) {
    if (n != 0) return;
    h = 0xcbf29ce484222325ull;
  } else {
    if (!live[slot]) return;
    h = fnv_bytes32(hash_in[(size_t)u * Wb + parent[slot]], (uint32_t)token[slot]);
  }
  if (threadIdx.x == 0) hash_out[slot] = h;
  make_row(stream_key(seed, TAG_ATT, (uint32_t)u, step, h), V, scale, 0.0, 0.0, -1, 0.0,
           out + (size_t)slot * V, logit, sh);
}

extern "C" int gen_dev_ctc(uint64_t seed, int n_utt, const int32_t* d_lens, int t_max, int V, int blank_id,
                           double boost, double p_boost, double zipf_s, float* d_out, void* stream) {
  double Z = 0.0;
  if (zipf_s > 0.0) for (int r = 1; r <= V - 1; ++r) Z += pow((double)r, -zipf_s);
  hipLaunchKernelGGL(k_gen_ctc, dim3(t_max, n_utt), dim3(256), sizeof(double) * (size_t)V, (hipStream_t)stream,
                     seed, d_lens, t_max, V, blank_id, boost, p_boost, zipf_s, zipf_s > 0.0 ? log(Z) : 0.0,
                     d_out);
  return (int)hipGetLastError();
}

extern "C" int gen_dev_att_step(uint64_t seed, uint32_t step, int n_utt, int Wb, int V, double scale,
                                const uint64_t* d_hash_in, const int32_t* d_parent, const int32_t* d_token,
                                const uint8_t* d_live, uint64_t* d_hash_out, float* d_out, void* stream) {
  hipLaunchKernelGGL(k_gen_att, dim3(n_utt * Wb), dim3(256), sizeof(double) * (size_t)V, (hipStream_t)stream,
                     seed, step, Wb, V, scale, step == 1 ? 1 : 0, d_hash_in, d_parent, d_token, d_live,
                     d_hash_out, d_out);
  return (int)hipGetLastError();
}
