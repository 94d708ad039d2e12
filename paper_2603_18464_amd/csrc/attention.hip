// Causal attention of single query rows against the KV cache.
//
// attention_rows: one wave per (token, head).  Lanes first split the keys (each lane scores keys
// lane, lane+64, ...), the softmax statistics are reduced across the wave, then lanes split the
// head dimension and accumulate the probability-weighted values.  Keys/values of a (slot, head)
// are contiguous [position][head_dim] rows in the cache.
#include "common.h"

namespace vla {

template <class T, int HD>
__global__ __launch_bounds__(256) void attention_rows_kernel(
    const T* __restrict__ q, int ldq, const T* __restrict__ k_cache, const T* __restrict__ v_cache,
    const int32_t* __restrict__ tok_seq, const int32_t* __restrict__ tok_pos, T* __restrict__ out, int ldo,
    int n_items, int n_heads, int max_seq) {
  extern __shared__ float smem[];                    // per wave: [HD] query + [max_seq] scores
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int item = blockIdx.x * 4 + wave;            // (token, head)
  if (item >= n_items) return;                       // whole wave leaves; no block barrier is used
  float* qs = smem + (size_t)wave * (HD + max_seq);
  float* sc = qs + HD;
  const int tok = item / n_heads, head = item - tok * n_heads;
  const int slot = tok_seq[tok], pos = tok_pos[tok];
  const int ctx = pos + 1;                           // keys 0..pos
  const T* qrow = q + (size_t)tok * ldq + head * HD;
  for (int i = lane; i < HD; i += 64) qs[i] = to_f32(qrow[i]);
  const T* kbase = k_cache + ((size_t)slot * n_heads + head) * max_seq * HD;
  const T* vbase = v_cache + ((size_t)slot * n_heads + head) * max_seq * HD;
  const float scale = rsqrtf((float)HD);
  __builtin_amdgcn_wave_barrier();
  float mx = -INFINITY;
  for (int key = lane; key < ctx; key += 64) {
    const T* kr = kbase + (size_t)key * HD;
    float s = 0.f;
#pragma unroll 8
    for (int i = 0; i < HD; ++i) s = fmaf(qs[i], to_f32(kr[i]), s);
    s *= scale;
    sc[key] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int key = lane; key < ctx; key += 64) {
    const float p = __expf(sc[key] - mx);
    sc[key] = p;
    sum += p;
  }
  sum = wave_sum(sum);
  __builtin_amdgcn_wave_barrier();
  const float inv = 1.0f / sum;
  T* orow = out + (size_t)tok * ldo + head * HD;
  for (int i = lane; i < HD; i += 64) {
    float acc = 0.f;
    for (int key = 0; key < ctx; ++key) acc = fmaf(sc[key], to_f32(vbase[(size_t)key * HD + i]), acc);
    orow[i] = from_f32<T>(acc * inv);
  }
}

template <class T>
void attention_rows(const T* q, int ldq, const T* k_cache, const T* v_cache, const int32_t* tok_seq,
                    const int32_t* tok_pos, T* out, int ldo, int n_tok, int n_heads, int head_dim, int max_seq,
                    hipStream_t st) {
  const int n_items = n_tok * n_heads;
  const int blocks = (n_items + 3) / 4;
  const size_t smem = 4 * (size_t)(head_dim + max_seq) * sizeof(float);
#define VLA_ATTN_CASE(HD)                                                                                   \
  case HD:                                                                                                  \
    hipLaunchKernelGGL((attention_rows_kernel<T, HD>), dim3(blocks), dim3(256), smem, st, q, ldq, k_cache,  \
                       v_cache, tok_seq, tok_pos, out, ldo, n_items, n_heads, max_seq);                     \
    break;
  switch (head_dim) {
    VLA_ATTN_CASE(32)
    VLA_ATTN_CASE(64)
    VLA_ATTN_CASE(128)
    VLA_ATTN_CASE(256)
    default: break;   // rejected by vla_create
  }
#undef VLA_ATTN_CASE
}
template void attention_rows<float>(const float*, int, const float*, const float*, const int32_t*, const int32_t*,
                                    float*, int, int, int, int, int, hipStream_t);
template void attention_rows<f16>(const f16*, int, const f16*, const f16*, const int32_t*, const int32_t*,
                                  f16*, int, int, int, int, int, hipStream_t);

}  // namespace vla
