// Row-wise and small kernels of the VLA policy path: prefix assembly, RMSNorm, the action head
// (final norm + slimmed LM head), token selection with log-probs and de-tokenisation, rotary
// tables, token maps, and the plain float32 path used when the storage dtype is float32.
#include "common.h"

namespace vla {

// ---- token maps ---------------------------------------------------------------------------------
// Packed prefix token t belongs to sequence b of the call with cu_seq[b] <= t < cu_seq[b+1], where
// cu_seq[b] = cu_patch[b] + cu_instr[b]; sequence b lives in cache slot slot_map[b] (b itself without a map).
// tok_src >= 0 is a row of patch_emb, tok_src < 0 is instruction id number -1 - tok_src.
__global__ void token_maps_kernel(const int32_t* __restrict__ cu_patch, const int32_t* __restrict__ cu_instr,
                                  const int32_t* __restrict__ slot_map, int B, int T, int32_t* tok_seq,
                                  int32_t* tok_pos, int32_t* tok_src, int32_t* last_row, int32_t* seq_len) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < B) {
    const int end = cu_patch[t + 1] + cu_instr[t + 1];
    last_row[t] = end - 1;
    seq_len[slot_map ? slot_map[t] : t] = end - (cu_patch[t] + cu_instr[t]);
  }
  if (t >= T) return;
  int lo = 0, hi = B;                       // find b with cu_seq[b] <= t < cu_seq[b+1]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu_patch[mid] + cu_instr[mid] <= t) lo = mid; else hi = mid;
  }
  const int b = lo;
  const int pos = t - (cu_patch[b] + cu_instr[b]);
  const int np = cu_patch[b + 1] - cu_patch[b];
  tok_seq[t] = slot_map ? slot_map[b] : b;
  tok_pos[t] = pos;
  tok_src[t] = pos < np ? cu_patch[b] + pos : -1 - (cu_instr[b] + pos - np);
}

void build_token_maps(const int32_t* cu_patch_dev, const int32_t* cu_instr_dev, const int32_t* slot_map, int B,
                      int T_tokens, int32_t* tok_seq, int32_t* tok_pos, int32_t* tok_src, int32_t* last_row,
                      int32_t* seq_len, hipStream_t st) {
  const int n = T_tokens > B ? T_tokens : B;
  hipLaunchKernelGGL(token_maps_kernel, dim3((n + 255) / 256), dim3(256), 0, st, cu_patch_dev, cu_instr_dev,
                     slot_map, B, T_tokens, tok_seq, tok_pos, tok_src, last_row, seq_len);
}

__global__ void decode_maps_kernel(const int32_t* seq_len, const int32_t* __restrict__ slot_map, int B,
                                   int32_t* tok_seq, int32_t* tok_pos) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) {
    const int slot = slot_map ? slot_map[b] : b;
    tok_seq[b] = slot;
    tok_pos[b] = seq_len[slot];
  }
}
void decode_maps(int32_t* seq_len, const int32_t* slot_map, int B, int32_t* tok_seq, int32_t* tok_pos, hipStream_t st) {
  hipLaunchKernelGGL(decode_maps_kernel, dim3((B + 255) / 256), dim3(256), 0, st, seq_len, slot_map, B, tok_seq,
                     tok_pos);
}

__global__ void advance_kernel(int32_t* seq_len, const int32_t* __restrict__ slot_map, int B) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) seq_len[slot_map ? slot_map[b] : b] += 1;
}
void advance_lengths(int32_t* seq_len, const int32_t* slot_map, int B, hipStream_t st) {
  hipLaunchKernelGGL(advance_kernel, dim3((B + 255) / 256), dim3(256), 0, st, seq_len, slot_map, B);
}

// ---- rotary table ---------------------------------------------------------------------------------
// cos/sin of pos * theta^(-2i/hd), evaluated in double so that the float32 path keeps 1e-4 logits.
__global__ void rope_table_kernel(float* cos_t, float* sin_t, int max_seq, int half, double theta) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= max_seq * half) return;
  const int pos = idx / half, i = idx - pos * half;
  const double inv = pow(theta, -(double)i / (double)half);
  const double ang = (double)pos * inv;
  cos_t[idx] = (float)cos(ang);
  sin_t[idx] = (float)sin(ang);
}
void rope_table(float* cos_t, float* sin_t, int max_seq, int head_dim, float theta, hipStream_t st) {
  const int n = max_seq * (head_dim / 2);
  hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, st, cos_t, sin_t, max_seq,
                     head_dim / 2, (double)theta);
}

// ---- copies ---------------------------------------------------------------------------------------
template <class T>
__global__ void convert_kernel(const T* src, float* dst, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = to_f32(src[i]);
}
template <class T>
void convert_copy(const T* src, float* dst, size_t n, hipStream_t st) {
  hipLaunchKernelGGL(convert_kernel<T>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, src, dst, n);
}
template void convert_copy<float>(const float*, float*, size_t, hipStream_t);
template void convert_copy<bf16>(const bf16*, float*, size_t, hipStream_t);

template <class T>
__global__ void copy_kernel(const T* src, T* dst, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = src[i];
}
template <class T>
void plain_copy(const T* src, T* dst, size_t n, hipStream_t st) {
  size_t blocks = (n + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(copy_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, st, src, dst, n);
}
template void plain_copy<float>(const float*, float*, size_t, hipStream_t);
template void plain_copy<bf16>(const bf16*, bf16*, size_t, hipStream_t);

// ---- prefix assembly ------------------------------------------------------------------------------
// x[t, :] = patch_emb[src] or embed[instr_ids[-1-src]], widened to the float32 residual stream.
template <class T>
__global__ void assemble_kernel(const T* __restrict__ patch_emb, const int32_t* __restrict__ instr_ids,
                                const T* __restrict__ embed, const int32_t* __restrict__ tok_src,
                                float* __restrict__ x, int d, int vocab) {
  const int t = blockIdx.x;
  const int src = tok_src[t];
  int id = src >= 0 ? 0 : instr_ids[-1 - src];
  id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);   // ids come from device memory: stay in bounds
  const T* row = src >= 0 ? patch_emb + (size_t)src * d : embed + (size_t)id * d;
  float* out = x + (size_t)t * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) out[i] = to_f32(row[i]);
}
template <class T>
void assemble_prefix(const T* patch_emb, const int32_t* instr_ids, const T* embed, const int32_t* tok_src,
                     float* x, int T_tokens, int d, int vocab, hipStream_t st) {
  hipLaunchKernelGGL(assemble_kernel<T>, dim3(T_tokens), dim3(256), 0, st, patch_emb, instr_ids, embed,
                     tok_src, x, d, vocab);
}
template void assemble_prefix<float>(const float*, const int32_t*, const float*, const int32_t*, float*, int,
                                     int, int, hipStream_t);
template void assemble_prefix<bf16>(const bf16*, const int32_t*, const bf16*, const int32_t*, float*, int, int,
                                    int, hipStream_t);

// ---- last-layer tail: only the rows that feed the head go through the last O / feed-forward ------------
// Row i of the compact set is packed row need[i]: its attention output goes to fragment order
// [i/32][k/16][lane][8] (what the weight-streaming GEMMs read), its residual row to x_c[i].
__global__ __launch_bounds__(256) void gather_tail_kernel(const f16* __restrict__ att, int ld_att, int lo8,
                                                          const float* __restrict__ x,
                                                          const int32_t* __restrict__ need, int d,
                                                          f16* __restrict__ att_frag, f16* __restrict__ att_frag_lo,
                                                          float* __restrict__ x_c) {
  const int i = blockIdx.x, src = need[i];
  const u32x4* arow = (const u32x4*)(att + (size_t)src * ld_att);
  u32x4* ablk = (u32x4*)(att_frag + (size_t)(i >> 5) * (d >> 4) * 512);
  for (int kc = threadIdx.x; kc < (d >> 3); kc += blockDim.x)
    ablk[(size_t)(kc >> 1) * 64 + (i & 31) + 32 * (kc & 1)] = arow[kc];
  if (att_frag_lo) {                       // two-term rows [hi | lo]: the low terms follow at column d
    u32x4* lblk = (u32x4*)(att_frag_lo + (size_t)(i >> 5) * (d >> 4) * 512);
    if (lo8) {                             // ... as bytes: widened to half precision (exact)
      const int* lrow = (const int*)(att + (size_t)src * ld_att + d);
      for (int kc = threadIdx.x; kc < (d >> 3); kc += blockDim.x) {
        const int w0 = lrow[2 * kc], w1 = lrow[2 * kc + 1];
        f16x8 h;
        h[0] = (f16)unpack_lo8(w0, 0); h[1] = (f16)unpack_lo8(w0, 1); h[2] = (f16)unpack_lo8(w0, 2); h[3] = (f16)unpack_lo8(w0, 3);
        h[4] = (f16)unpack_lo8(w1, 0); h[5] = (f16)unpack_lo8(w1, 1); h[6] = (f16)unpack_lo8(w1, 2); h[7] = (f16)unpack_lo8(w1, 3);
        lblk[(size_t)(kc >> 1) * 64 + (i & 31) + 32 * (kc & 1)] = __builtin_bit_cast(u32x4, h);
      }
    } else {
      const u32x4* lrow = (const u32x4*)(att + (size_t)src * ld_att + d);
      for (int kc = threadIdx.x; kc < (d >> 3); kc += blockDim.x)
        lblk[(size_t)(kc >> 1) * 64 + (i & 31) + 32 * (kc & 1)] = lrow[kc];
    }
  }
  const f32x4* xr = (const f32x4*)(x + (size_t)src * d);
  f32x4* xo = (f32x4*)(x_c + (size_t)i * d);
  for (int j = threadIdx.x; j < (d >> 2); j += blockDim.x) xo[j] = xr[j];
}
void gather_tail(const f16* att, int ld_att, bool lo8, const float* x, const int32_t* need, int n, int d,
                 f16* att_frag, f16* att_frag_lo, float* x_c, hipStream_t st) {
  hipLaunchKernelGGL(gather_tail_kernel, dim3(n), dim3(256), 0, st, att, ld_att, lo8 ? 1 : 0, x, need, d, att_frag,
                     att_frag_lo, x_c);
}
__global__ __launch_bounds__(256) void scatter_tail_kernel(const float* __restrict__ x_c,
                                                           const int32_t* __restrict__ need, int d,
                                                           float* __restrict__ x) {
  const int i = blockIdx.x;
  const f32x4* xr = (const f32x4*)(x_c + (size_t)i * d);
  f32x4* xo = (f32x4*)(x + (size_t)need[i] * d);
  for (int j = threadIdx.x; j < (d >> 2); j += blockDim.x) xo[j] = xr[j];
}
void scatter_tail(const float* x_c, const int32_t* need, int n, int d, float* x, hipStream_t st) {
  hipLaunchKernelGGL(scatter_tail_kernel, dim3(n), dim3(256), 0, st, x_c, need, d, x);
}

// ---- chunk pass: every sequence is [prefix ; n_tail fed tokens], logits wanted at its last n_tail + 1 rows ----
// cu2[b] = cu_instr[b] + b * n_tail are the offsets of the merged id stream.
__global__ void merge_tail_kernel(const int32_t* __restrict__ instr_ids, const int32_t* __restrict__ cu2,
                                  const int32_t* __restrict__ tail, int B, int n_tail, int total,
                                  int32_t* __restrict__ out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  int lo = 0, hi = B;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu2[mid] <= i) lo = mid; else hi = mid;
  }
  const int b = lo, j = i - cu2[b];
  const int li = cu2[b + 1] - cu2[b] - n_tail;
  out[i] = j < li ? instr_ids[cu2[b] - b * n_tail + j] : tail[b * n_tail + (j - li)];
}
void merge_tail_ids(const int32_t* instr_ids, const int32_t* cu2_dev, const int32_t* tail, int B, int n_tail,
                    int total, int32_t* out, hipStream_t st) {
  if (total <= 0) return;
  hipLaunchKernelGGL(merge_tail_kernel, dim3((total + 255) / 256), dim3(256), 0, st, instr_ids, cu2_dev, tail, B,
                     n_tail, total, out);
}

// tail[b, j] = placeholder (tokens == nullptr) or the vocabulary id of stored bin tokens[b, j], j < K - 1
__global__ void tail_ids_kernel(const int32_t* __restrict__ tokens, int B, int K, int id0, int A, int placeholder,
                                int32_t* __restrict__ tail) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B * (K - 1)) return;
  const int b = i / (K - 1), j = i - b * (K - 1);
  if (tokens) {
    int t = tokens[b * K + j];
    t = t < 0 ? 0 : (t >= A ? A - 1 : t);
    tail[i] = id0 + t;
  } else {
    tail[i] = placeholder;
  }
}
void tail_ids(const int32_t* tokens, int B, int K, int id0, int A, int placeholder, int32_t* tail, hipStream_t st) {
  const int n = B * (K - 1);
  if (n <= 0) return;
  hipLaunchKernelGGL(tail_ids_kernel, dim3((n + 255) / 256), dim3(256), 0, st, tokens, B, K, id0, A, placeholder, tail);
}

// rows[b * K + k] = packed row that emits action token k of sequence b
__global__ void chunk_rows_kernel(const int32_t* __restrict__ last_row, int B, int K, int32_t* __restrict__ rows) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B * K) return;
  const int b = i / K, k = i - b * K;
  rows[i] = last_row[b] - (K - 1) + k;
}
void chunk_rows(const int32_t* last_row, int B, int K, int32_t* rows, hipStream_t st) {
  hipLaunchKernelGGL(chunk_rows_kernel, dim3((B * K + 255) / 256), dim3(256), 0, st, last_row, B, K, rows);
}

// One wave per (sequence, token): log-prob of a given bin under log_softmax(logits / tau), and with the
// behaviour log-prob mu the importance ratio rho = exp(logp - mu) and rho * exp(-(log rho / sigma)^2 / 2).
__global__ __launch_bounds__(64) void score_kernel(const float* __restrict__ logits, int A, float temperature,
                                                   const int32_t* __restrict__ tokens,
                                                   const float* __restrict__ mu, float sigma,
                                                   float* __restrict__ logp_out, float* __restrict__ ratio_out,
                                                   float* __restrict__ weight_out) {
  const int r = blockIdx.x, lane = threadIdx.x;
  const float* z = logits + (size_t)r * A;
  const float inv_tau = temperature > 0.f ? 1.0f / temperature : 1.0f;
  float zmax = -INFINITY;
  for (int j = lane; j < A; j += 64) zmax = fmaxf(zmax, z[j] * inv_tau);
  zmax = wave_max(zmax);
  float se = 0.f;
  for (int j = lane; j < A; j += 64) se += expf(z[j] * inv_tau - zmax);
  se = wave_sum(se);
  if (lane == 0) {
    int t = tokens[r];
    t = t < 0 ? 0 : (t >= A ? A - 1 : t);
    const float logp = z[t] * inv_tau - zmax - logf(se);
    logp_out[r] = logp;
    if (mu) {
      const float lr = logp - mu[r];
      const float rho = expf(lr);
      const float q = lr / sigma;
      if (ratio_out) ratio_out[r] = rho;
      if (weight_out) weight_out[r] = rho * expf(-0.5f * q * q);
    }
  }
}
void score_rows(const float* logits, int rows, int A, float temperature, const int32_t* tokens, const float* mu,
                float sigma, float* logp_out, float* ratio_out, float* weight_out, hipStream_t st) {
  hipLaunchKernelGGL(score_kernel, dim3(rows), dim3(64), 0, st, logits, A, temperature, tokens, mu, sigma, logp_out,
                     ratio_out, weight_out);
}

template <class T>
__global__ void embed_kernel(const int32_t* __restrict__ ids, const T* __restrict__ embed,
                             float* __restrict__ x, int d, int vocab) {
  const int b = blockIdx.x;
  int id = ids[b];
  id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);   // ids come from device memory: stay in bounds
  const T* row = embed + (size_t)id * d;
  float* out = x + (size_t)b * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) out[i] = to_f32(row[i]);
}
template <class T>
void embed_tokens(const int32_t* ids, const T* embed, float* x, int B, int d, int vocab, hipStream_t st) {
  hipLaunchKernelGGL(embed_kernel<T>, dim3(B), dim3(256), 0, st, ids, embed, x, d, vocab);
}
template void embed_tokens<float>(const int32_t*, const float*, float*, int, int, int, hipStream_t);
template void embed_tokens<bf16>(const int32_t*, const bf16*, float*, int, int, int, hipStream_t);

// ---- RMSNorm ----------------------------------------------------------------------------------------
// out[r, :] = x[row, :] * gain / sqrt(mean(x^2) + eps), statistics in float32; one workgroup per row.
__device__ __forceinline__ float block_sum_256(float v, float* red) {
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

template <class T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ x, const float* __restrict__ gain,
                                                      T* __restrict__ out, int d, float eps,
                                                      const int32_t* __restrict__ row_index, int ldo, int lo_mode) {
  typedef __attribute__((ext_vector_type(4))) T T4;
  __shared__ float red[4];
  const int r = blockIdx.x;
  const float* row = x + (size_t)(row_index ? row_index[r] : r) * d;
  constexpr int kHeld = 8;                 // float4 per thread kept in registers: rows up to 8192 wide are read once
  f32x4 held[kHeld];
  float ss = 0.f;
#pragma unroll
  for (int it = 0; it < kHeld; ++it) {
    const int i = threadIdx.x * 4 + it * 1024;
    held[it] = i < d ? *(const f32x4*)(row + i) : f32x4{0.f, 0.f, 0.f, 0.f};
    ss += held[it][0] * held[it][0] + held[it][1] * held[it][1] + held[it][2] * held[it][2] + held[it][3] * held[it][3];
  }
  for (int i = threadIdx.x * 4 + kHeld * 1024; i < d; i += 1024) {
    const f32x4 v = *(const f32x4*)(row + i);
    ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
  }
  ss = block_sum_256(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  T* o = out + (size_t)r * ldo;
  // lo_mode 1 (two-term output): the low terms go to column d + i; 2: as bytes behind the d high terms
  auto emit = [&](int i, const f32x4& v) {
    const f32x4 g = *(const f32x4*)(gain + i);
    T4 q, qe;
    float e[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float h = v[j] * inv * g[j];
      q[j] = from_f32<T>(h);
      e[j] = h - to_f32(q[j]);
      qe[j] = from_f32<T>(e[j]);
    }
    *(T4*)(o + i) = q;
    if (lo_mode == 1) *(T4*)(o + d + i) = qe;
    if (lo_mode == 2) *(int*)((unsigned char*)(o + d) + i) = pack_lo8(e[0], e[1], e[2], e[3]);
  };
#pragma unroll
  for (int it = 0; it < kHeld; ++it) {
    const int i = threadIdx.x * 4 + it * 1024;
    if (i < d) emit(i, held[it]);
  }
  for (int i = threadIdx.x * 4 + kHeld * 1024; i < d; i += 1024) emit(i, *(const f32x4*)(row + i));
}
template <class T>
void rmsnorm(const float* x, const T*, const float* gain, T* out, int rows, int d, float eps,
             const int32_t* row_index, int lo_mode, hipStream_t st) {
  hipLaunchKernelGGL(rmsnorm_kernel<T>, dim3(rows), dim3(256), 0, st, x, gain, out, d, eps, row_index,
                     lo_mode == 1 ? 2 * d : (lo_mode == 2 ? d + d / 2 : d), lo_mode);
}
template void rmsnorm<float>(const float*, const float*, const float*, float*, int, int, float, const int32_t*,
                             int, hipStream_t);
template void rmsnorm<f16>(const float*, const f16*, const float*, f16*, int, int, float, const int32_t*,
                           int, hipStream_t);

// ---- action head ------------------------------------------------------------------------------------
// Workgroup (b, g): final RMSNorm of sequence b's row (float32, kept in LDS), then 32 action rows of
// the slimmed head, 8 per wave, lanes striding over d with a wave reduction per row.  The norm is
// recomputed by each of the A/32 workgroups of a sequence: that is 16 KiB from L2, and it spreads the
// head over B * A/32 workgroups instead of B.
constexpr int kHeadRows = 32;
template <class T>
__global__ __launch_bounds__(256) void head_kernel(const float* __restrict__ x, const int32_t* __restrict__ row_index,
                                                   const float* __restrict__ gain, const T* __restrict__ w_head,
                                                   float* __restrict__ logits, int ld_logits, int d, int A, float eps) {
  extern __shared__ float hrow[];          // [d]
  __shared__ float red[4];
  const int b = blockIdx.x;
  const float* row = x + (size_t)(row_index ? row_index[b] : b) * d;
  float ss = 0.f;
  for (int i = threadIdx.x * 4; i < d; i += 1024) {
    const float4 v = *(const float4*)(row + i);
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ss = block_sum_256(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  for (int i = threadIdx.x * 4; i < d; i += 1024) {
    const float4 v = *(const float4*)(row + i);
    const float4 g = *(const float4*)(gain + i);
    *(float4*)(hrow + i) = make_float4(v.x * inv * g.x, v.y * inv * g.y, v.z * inv * g.z, v.w * inv * g.w);
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j0 = blockIdx.y * kHeadRows;
  for (int j = j0 + wave; j < min(j0 + kHeadRows, A); j += 4) {
    const T* w = w_head + (size_t)j * d;
    float acc = 0.f;
    for (int i = lane * 4; i < d; i += 256) {
      const float4 h = *(const float4*)(hrow + i);
      acc += to_f32(w[i]) * h.x + to_f32(w[i + 1]) * h.y + to_f32(w[i + 2]) * h.z + to_f32(w[i + 3]) * h.w;
    }
    acc = wave_sum(acc);
    if (lane == 0) logits[(size_t)b * ld_logits + j] = acc;
  }
}
template <class T>
void head_logits(const float* x, const int32_t* row_index, const float* gain, const T* w_head, float* logits,
                 int ld_logits, int B, int d, int A, float eps, hipStream_t st) {
  hipLaunchKernelGGL(head_kernel<T>, dim3(B, (A + kHeadRows - 1) / kHeadRows), dim3(256), d * sizeof(float), st, x,
                     row_index, gain, w_head, logits, ld_logits, d, A, eps);
}
template void head_logits<float>(const float*, const int32_t*, const float*, const float*, float*, int, int, int,
                                 int, float, hipStream_t);
template void head_logits<bf16>(const float*, const int32_t*, const float*, const bf16*, float*, int, int, int,
                                int, float, hipStream_t);

// ---- value head ---------------------------------------------------------------------------------------
// Action-aware attention pooling over the K hidden rows that feed the action head, done online: after
// each head evaluation the row's score e = w_attn . h + b_attn updates a running softmax-weighted sum
// (m, l, z) per sequence, so no hidden state is stored.  h is the final-RMSNorm output in float32.
__global__ __launch_bounds__(256) void value_accumulate_kernel(const float* __restrict__ x,
                                                               const int32_t* __restrict__ row_index,
                                                               const float* __restrict__ gain, float eps,
                                                               const float* __restrict__ attn_w,
                                                               const float* __restrict__ attn_b, int d, int first,
                                                               float* __restrict__ vz, float* __restrict__ vml) {
  __shared__ float red[4];
  const int b = blockIdx.x;
  const float* row = x + (size_t)(row_index ? row_index[b] : b) * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) ss += row[i] * row[i];
  ss = block_sum_256(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  float e = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) e += row[i] * inv * gain[i] * attn_w[i];
  e = block_sum_256(e, red) + attn_b[0];
  const float m_old = first ? -INFINITY : vml[2 * b], l_old = first ? 0.f : vml[2 * b + 1];
  const float m_new = fmaxf(m_old, e);
  const float scale = first ? 0.f : expf(m_old - m_new), p = expf(e - m_new);
  float* z = vz + (size_t)b * d;
  for (int i = threadIdx.x; i < d; i += 256) {
    const float h = row[i] * inv * gain[i];
    z[i] = (first ? 0.f : z[i] * scale) + p * h;
  }
  __syncthreads();                       // every thread has read the old statistics
  if (threadIdx.x == 0) {
    vml[2 * b] = m_new;
    vml[2 * b + 1] = l_old * scale + p;
  }
}
void value_accumulate(const float* x, const int32_t* row_index, const float* gain, float eps, const float* attn_w,
                      const float* attn_b, int B, int d, bool first, float* vz, float* vml, hipStream_t st) {
  hipLaunchKernelGGL(value_accumulate_kernel, dim3(B), dim3(256), 0, st, x, row_index, gain, eps, attn_w, attn_b, d,
                     first ? 1 : 0, vz, vml);
}

// u[b] = z[b] / l[b] + step_emb[step_t[b]]   (step clamped to the table)
template <class T>
__global__ __launch_bounds__(256) void value_pool_kernel(const float* __restrict__ vz, const float* __restrict__ vml,
                                                         const T* __restrict__ step_emb, int n_steps,
                                                         const int32_t* __restrict__ step_t, int d,
                                                         float* __restrict__ vu) {
  const int b = blockIdx.x;
  int t = step_t[b];
  t = t < 0 ? 0 : (t >= n_steps ? n_steps - 1 : t);
  const float inv_l = 1.0f / vml[2 * b + 1];
  for (int i = threadIdx.x; i < d; i += 256)
    vu[(size_t)b * d + i] = vz[(size_t)b * d + i] * inv_l + to_f32(step_emb[(size_t)t * d + i]);
}

// vh[b][j] = w2[j] * gelu(W1[j,:] . u[b] + b1[j]).  A workgroup keeps RB rows of u in LDS; each wave then walks
// 16 rows of W1, reading every weight once from memory for all RB rows.
__device__ __forceinline__ f32x4 load4_f32(const float* p) { return *(const f32x4*)p; }
__device__ __forceinline__ f32x4 load4_f32(const bf16* p) {
  const bf16x4 v = *(const bf16x4*)p;
  return f32x4{(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
}
template <class T, int RB>
__global__ __launch_bounds__(256) void value_mlp_kernel(const T* __restrict__ w1, const float* __restrict__ b1,
                                                        const float* __restrict__ w2, const float* __restrict__ vu,
                                                        int B, int d, float* __restrict__ vh) {
  extern __shared__ float us[];                             // [RB][d]
  constexpr int JPW = 16;                                   // rows of W1 per wave
  const int b0 = blockIdx.x * RB, nb = min(RB, B - b0);
  for (int i = threadIdx.x * 4; i < RB * d; i += 1024) {
    const int r = i / d, c = i - r * d;                     // d is a multiple of 4: a float4 stays inside a row
    *(f32x4*)(us + i) = r < nb ? *(const f32x4*)(vu + (size_t)(b0 + r) * d + c) : f32x4{0.f, 0.f, 0.f, 0.f};
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int jj = 0; jj < JPW; ++jj) {
    const int j = (blockIdx.y * 4 + wave) * JPW + jj;
    if (j >= d) break;                                      // uniform per wave
    const T* wr = w1 + (size_t)j * d;
    float acc[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) acc[r] = 0.f;
    for (int c = lane * 4; c < d; c += 256) {
      const f32x4 w = load4_f32(wr + c);
#pragma unroll
      for (int r = 0; r < RB; ++r) {
        const f32x4 u = *(const f32x4*)(us + r * d + c);
        acc[r] += w[0] * u[0] + w[1] * u[1] + w[2] * u[2] + w[3] * u[3];
      }
    }
#pragma unroll
    for (int r = 0; r < RB; ++r) acc[r] = wave_sum(acc[r]);
    if (lane == 0) {
      const float bj = b1[j], wj = w2[j];
#pragma unroll
      for (int r = 0; r < RB; ++r)
        if (r < nb) {
          const float t = acc[r] + bj;
          vh[(size_t)(b0 + r) * d + j] = wj * 0.5f * t * (1.0f + erff(t * 0.70710678118654752f));
        }
    }
  }
}
template <class T, int RB>
static void launch_value_mlp(const T* w1, const float* b1, const float* w2, const float* vu, int B, int d, float* vh,
                             hipStream_t st) {
  const size_t smem = (size_t)RB * d * sizeof(float);
  auto kern = value_mlp_kernel<T, RB>;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3((B + RB - 1) / RB, (d + 63) / 64), dim3(256), smem, st, w1, b1, w2, vu, B, d, vh);
}

__global__ __launch_bounds__(256) void value_sum_kernel(const float* __restrict__ vh, const float* __restrict__ b2,
                                                        int d, float* __restrict__ values) {
  __shared__ float red[4];
  const int b = blockIdx.x;
  float s = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) s += vh[(size_t)b * d + i];
  s = block_sum_256(s, red);
  if (threadIdx.x == 0) values[b] = s + b2[0];
}

template <class T>
void value_finish(const float* vz, const float* vml, const T* step_emb, int n_steps, const int32_t* step_t,
                  const T* w1, const float* b1, const float* w2, const float* b2, int B, int d, float* vu, float* vh,
                  float* values, hipStream_t st) {
  hipLaunchKernelGGL(value_pool_kernel<T>, dim3(B), dim3(256), 0, st, vz, vml, step_emb, n_steps, step_t, d, vu);
  if (d <= 5120) launch_value_mlp<T, 8>(w1, b1, w2, vu, B, d, vh, st);            // RB * d floats of LDS <= 160 KiB
  else if (d <= 10240) launch_value_mlp<T, 4>(w1, b1, w2, vu, B, d, vh, st);
  else launch_value_mlp<T, 2>(w1, b1, w2, vu, B, d, vh, st);
  hipLaunchKernelGGL(value_sum_kernel, dim3(B), dim3(256), 0, st, vh, b2, d, values);
}
template void value_finish<float>(const float*, const float*, const float*, int, const int32_t*, const float*,
                                  const float*, const float*, const float*, int, int, float*, float*, float*,
                                  hipStream_t);
template void value_finish<bf16>(const float*, const float*, const bf16*, int, const int32_t*, const bf16*,
                                 const float*, const float*, const float*, int, int, float*, float*, float*,
                                 hipStream_t);

// ---- practical ceilings, measured on request ------------------------------------------------------------
// MFMA-only loop: every wave loads two A and four B fragments once (real weight bits, so the operands toggle
// like real data) and issues 8 independent 32x32x16 MFMAs per iteration on them; nothing else runs.
__global__ __launch_bounds__(256) void probe_mfma_kernel(const f16* __restrict__ w, size_t n_frag, int iters,
                                                         float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  f16x8 a[2], b[4];
#pragma unroll
  for (int i = 0; i < 2; ++i) a[i] = *(const f16x8*)(w + ((wave * 6 + i) % n_frag) * 512 + lane * 8);
#pragma unroll
  for (int i = 0; i < 4; ++i) b[i] = *(const f16x8*)(w + ((wave * 6 + 2 + i) % n_frag) * 512 + lane * 8);
  f32x16 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  for (int it = 0; it < iters; ++it)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) t += acc[i][j][0];
  if (t == 123.456f) sink[0] = t;      // keeps the loop alive; never true in practice
}
void probe_mfma(const f16* w, size_t n_frag, int n_wg, int iters, float* sink, hipStream_t st) {
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(n_wg), dim3(256), 0, st, w, n_frag, iters, sink);
}
// Streaming read: 16 bytes per lane, grid-stride, four loads in flight per lane.
__global__ __launch_bounds__(256) void probe_stream_kernel(const u32x4* __restrict__ src, size_t n16,
                                                           unsigned* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  unsigned x = 0;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const u32x4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    x ^= a[0] ^ b[1] ^ c[2] ^ d[3];
  }
  for (; i < n16; i += stride) x ^= src[i][0];
  if (x == 0x9e3779b9u) sink[0] = x;   // practically never
}
void probe_stream(const void* src, size_t bytes, int n_wg, unsigned* sink, hipStream_t st) {
  hipLaunchKernelGGL(probe_stream_kernel, dim3(n_wg), dim3(256), 0, st, (const u32x4*)src, bytes / 16, sink);
}

// ---- selection ----------------------------------------------------------------------------------------
// One wave per sequence: scores = logits / tau (+ Gumbel noise); token = lowest index among the
// maxima; log-prob = log_softmax(logits / tau)[token]; action = bin centre (optionally affine).
// Non-finite input: NaN scores never win the comparison, so the token is the best of the others; a row
// with no score above -inf (all NaN or all -inf) selects bin 0.  The log-prob of such rows is NaN.
__global__ __launch_bounds__(64) void select_kernel(const float* __restrict__ logits, int ld_logits, int A, float temperature,
                                                    const float* __restrict__ gumbel, int k, int n_tokens,
                                                    const float* __restrict__ act_scale,
                                                    const float* __restrict__ act_offset, int action_dim,
                                                    int32_t* tokens_out, float* logp_out, float* actions_out,
                                                    int out_stride, int32_t* next_ids, int id0) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const float* z = logits + (size_t)b * ld_logits;
  const float inv_tau = temperature > 0.f ? 1.0f / temperature : 1.0f;
  const float* g = (gumbel && temperature > 0.f) ? gumbel + ((size_t)b * n_tokens + k) * A : nullptr;
  float best = -INFINITY, zmax = -INFINITY;
  int best_j = 0x7fffffff;
  for (int j = lane; j < A; j += 64) {
    const float y = z[j] * inv_tau;
    const float s = g ? y + g[j] : y;
    if (s > best) { best = s; best_j = j; }      // strict: keeps the lowest index within a lane
    zmax = fmaxf(zmax, y);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ob = __shfl_xor(best, o, 64);
    const int oj = __shfl_xor(best_j, o, 64);
    if (ob > best || (ob == best && oj < best_j)) { best = ob; best_j = oj; }
  }
  if (best_j >= A) best_j = 0;                     // no lane saw a score above -inf
  zmax = wave_max(zmax);
  float se = 0.f;
  for (int j = lane; j < A; j += 64) se += expf(z[j] * inv_tau - zmax);
  se = wave_sum(se);
  if (lane == 0) {
    const float logp = z[best_j] * inv_tau - zmax - logf(se);
    float a = -1.0f + (2.0f * (float)best_j + 1.0f) / (float)A;
    const int dim = action_dim > 0 ? k % action_dim : 0;
    if (act_scale) a *= act_scale[dim];
    if (act_offset) a += act_offset[dim];
    const size_t o = (size_t)b * out_stride + k;
    tokens_out[o] = best_j;
    logp_out[o] = logp;
    actions_out[o] = a;
    if (next_ids) next_ids[b] = id0 + best_j;
  }
}
void select_tokens(const float* logits, int ld_logits, int B, int A, float temperature, const float* gumbel, int k, int n_tokens,
                   const float* act_scale, const float* act_offset, int action_dim, int32_t* tokens_out,
                   float* logp_out, float* actions_out, int out_stride, int32_t* next_ids, int id0,
                   hipStream_t st) {
  hipLaunchKernelGGL(select_kernel, dim3(B), dim3(64), 0, st, logits, ld_logits, A, temperature, gumbel, k, n_tokens,
                     act_scale, act_offset, action_dim, tokens_out, logp_out, actions_out, out_stride, next_ids,
                     id0);
}

// ---- float32 path -------------------------------------------------------------------------------------
// C[M,N] = A[M,K] * W[N,K]^T, 64x64 tiles, 16-deep K slabs in LDS, 4x4 outputs per thread.
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, int lda,
                                                       const float* __restrict__ W, float* __restrict__ C, int M,
                                                       int N, int K) {
  __shared__ float As[16][64 + 1];
  __shared__ float Ws[16][64 + 1];
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int i = threadIdx.x; i < 64 * 16; i += 256) {
      const int r = i >> 4, kk = i & 15;
      const int gm = m0 + r, gn = n0 + r, gk = k0 + kk;
      As[kk][r] = (gm < M && gk < K) ? A[(size_t)gm * lda + gk] : 0.f;
      Ws[kk][r] = (gn < N && gk < K) ? W[(size_t)gn * K + gk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) w[j] = Ws[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < M && n < N) C[(size_t)m * N + n] = acc[i][j];
    }
}
void gemm_f32(const float* A, int lda, const float* W, float* C, int M, int N, int K, hipStream_t st) {
  hipLaunchKernelGGL(gemm_f32_kernel, dim3((N + 63) / 64, (M + 63) / 64), dim3(256), 0, st, A, lda, W, C, M, N, K);
}

// qkv [T, 3d] float32 -> rotated q [T, d], rotated k and plain v into the cache.
__global__ void rope_kv_f32_kernel(const float* __restrict__ qkv, RopeKv o) {
  const int t = blockIdx.x;
  const int d = o.d_model, hd = o.head_dim, half = hd >> 1;
  const int pos = o.tok_pos[t], slot = o.tok_seq[t];
  const float* row = qkv + (size_t)t * 3 * d;
  for (int idx = threadIdx.x; idx < d / 2; idx += blockDim.x) {
    const int head = idx / half, i = idx - head * half;
    const float cs = o.rope_cos[pos * half + i], sn = o.rope_sin[pos * half + i];
    const int c0 = head * hd + i, c1 = c0 + half;
    const size_t kv = (((size_t)slot * o.n_heads + head) * o.max_seq + pos) * hd;
    const float q0 = row[c0], q1 = row[c1], k0 = row[d + c0], k1 = row[d + c1];
    float* q = (float*)o.q + (size_t)t * d;
    q[c0] = q0 * cs - q1 * sn;
    q[c1] = q1 * cs + q0 * sn;
    ((float*)o.k_cache)[kv + i] = k0 * cs - k1 * sn;
    ((float*)o.k_cache)[kv + i + half] = k1 * cs + k0 * sn;
    ((float*)o.v_cache)[kv + i] = row[2 * d + c0];
    ((float*)o.v_cache)[kv + i + half] = row[2 * d + c1];
  }
}
void rope_kv_f32(const float* qkv, int T, const RopeKv& o, hipStream_t st) {
  hipLaunchKernelGGL(rope_kv_f32_kernel, dim3(T), dim3(128), 0, st, qkv, o);
}

__global__ void resid_add_kernel(float* x, const float* c, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) x[i] += c[i];
}
void resid_add_f32(float* x, const float* c, size_t n, hipStream_t st) {
  hipLaunchKernelGGL(resid_add_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, x, c, n);
}

// gu [T, 2f] = [gate | up] -> act [T, f] = silu(gate) * up
__global__ void swiglu_f32_kernel(const float* __restrict__ gu, float* __restrict__ act, int f, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const size_t t = i / f;
  const int j = (int)(i - t * f);
  const float g = gu[t * 2 * f + j], u = gu[t * 2 * f + f + j];
  act[i] = g / (1.0f + expf(-g)) * u;
}
void swiglu_f32(const float* gu, float* act, int T, int f, hipStream_t st) {
  const size_t n = (size_t)T * f;
  hipLaunchKernelGGL(swiglu_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, gu, act, f, n);
}

}  // namespace vla
