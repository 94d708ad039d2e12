// Decode-step GEMMs: C[M,N] = A[M,K] * W[N,K]^T with M = batch (<= 128 rows), bound by streaming the
// weights from HBM once.  No LDS and no barriers in the streaming loop: every wave is an independent
// stream.
//
//   * A wave owns two 32-row weight blocks (64 output columns) over one slice of K.  Per k-step of 16
//     it loads two weight fragments (1 KiB each, fully coalesced, straight from the packed layout into
//     MFMA operand registers) and M/32 activation fragments, and issues 2*M/32 MFMAs.
//   * Activations are kept in the same fragment order as the weights ([m/32][k/16][lane][8], written
//     that way by the producing kernels), so their loads are coalesced 1 KiB reads that hit in L2.
//   * Loads run D k-steps ahead of the MFMAs through a register ring (static indices after unrolling),
//     which keeps D * (2 + M/32) KiB per wave in flight.
//   * K is split into 4 * kgroups slices to put enough waves on the chip.  The four waves of a
//     workgroup add their partial tiles through LDS; one plane part[kg][M][N] is written per group and
//     the following reduce kernel adds the planes in a fixed order (deterministic) and applies the
//     layer's elementwise step: RoPE + KV append, residual add + RMSNorm for the next GEMM, or SwiGLU.
#include "common.h"

namespace vla {

template <int MT, int D>
__global__ __launch_bounds__(256) void skinny_gemm_kernel(const f16* __restrict__ Af, const f16* __restrict__ Wp,
                                                          float* __restrict__ part, int M, int N, int K,
                                                          int kgroups) {
  // Workgroup = one pair of 32-row weight blocks (64 output columns) x one group of 4 K slices; wave w
  // streams slice 4*kg + w.  The four partial tiles are added through LDS in the fixed order
  // (w0 + w2) + (w1 + w3), so one plane part[kg] is written per group, deterministically.
  extern __shared__ float red[];                          // [2][MT*32 regs][64 lanes]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int NP = N >> 6;
  const int nbp = blockIdx.x % NP, kg = blockIdx.x / NP;
  const int KB16 = K >> 4;
  const int slices = 4 * kgroups, sl = 4 * kg + wave;
  const int kb_begin = (int)((long long)sl * KB16 / slices);
  const int kb_end = (int)((long long)(sl + 1) * KB16 / slices);   // non-empty: slices <= KB16

  const f16* w0 = Wp + ((size_t)(2 * nbp) * KB16) * 512 + lane * 8;
  const f16* w1 = w0 + (size_t)KB16 * 512;
  const f16* a0 = Af + lane * 8;

  f32x16 acc[MT][2];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // Each wave walks its slice from a different starting point (rotated by its column pair).  The rows of
  // the packed matrix are a power-of-two number of bytes apart for K = 4096, so waves marching through k
  // in lockstep would all hit the same memory channels at the same time.
  const int len = kb_end - kb_begin;
  const int rot = (nbp * 5) % len;
  auto kb_of = [&](int i) {                                // i-th step of this wave, clamped to the slice
    const int j = min(i, len - 1) + rot;
    return (size_t)(kb_begin + (j >= len ? j - len : j));
  };
  f16x8 wq[D][2], aq[D][MT];
#pragma unroll
  for (int s = 0; s < D; ++s) {
    const size_t kb = kb_of(s);
    wq[s][0] = *(const f16x8*)(w0 + kb * 512);
    wq[s][1] = *(const f16x8*)(w1 + kb * 512);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) aq[s][mt] = *(const f16x8*)(a0 + ((size_t)mt * KB16 + kb) * 512);
  }
  // Full groups of D k-steps: straight-line body (no branches, so the load counter is tracked exactly and
  // each MFMA waits only for its own stage); every consumed stage is refilled D steps ahead, clamped to the
  // last step of the slice.  The remaining steps (< D) sit in the first stages after the last group.
  const int n_full = len / D;
  for (int g = 0; g < n_full; ++g) {
    const int base = g * D;
#pragma unroll
    for (int s = 0; s < D; ++s) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        acc[mt][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aq[s][mt], wq[s][0], acc[mt][0], 0, 0, 0);
        acc[mt][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aq[s][mt], wq[s][1], acc[mt][1], 0, 0, 0);
      }
      const size_t kb = kb_of(base + s + D);
      wq[s][0] = *(const f16x8*)(w0 + kb * 512);
      wq[s][1] = *(const f16x8*)(w1 + kb * 512);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) aq[s][mt] = *(const f16x8*)(a0 + ((size_t)mt * KB16 + kb) * 512);
      __builtin_amdgcn_sched_barrier(0);   // keep the refills in stage order, or the oldest stage's wait
                                           // degenerates into a wait for every outstanding load
    }
  }
  const int rem = len - n_full * D;
#pragma unroll
  for (int s = 0; s < D; ++s) {
    if (s < rem) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        acc[mt][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aq[s][mt], wq[s][0], acc[mt][0], 0, 0, 0);
        acc[mt][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aq[s][mt], wq[s][1], acc[mt][1], 0, 0, 0);
      }
    }
  }
  // tree reduction over the four waves
  constexpr int REGS = MT * 32;
  auto put = [&](int slot) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) red[((size_t)slot * REGS + (mt * 2 + j) * 16 + e) * 64 + lane] = acc[mt][j][e];
  };
  auto add = [&](int slot) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[mt][j][e] += red[((size_t)slot * REGS + (mt * 2 + j) * 16 + e) * 64 + lane];
  };
  if (wave >= 2) put(wave - 2);
  __syncthreads();
  if (wave < 2) add(wave);                                  // w0 += w2, w1 += w3
  __syncthreads();
  if (wave == 1) put(0);
  __syncthreads();
  if (wave != 0) return;
  add(0);
  const int h = lane >> 5, c = lane & 31;
  float* out = part + (size_t)kg * M * N + nbp * 64 + c;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int blk = 0; blk < 4; ++blk)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = mt * 32 + 8 * blk + 4 * h + r;
        if (m < M) {
          out[(size_t)m * N] = acc[mt][0][4 * blk + r] * (1.0f / kWeightScale);
          out[(size_t)m * N + 32] = acc[mt][1][4 * blk + r] * (1.0f / kWeightScale);
        }
      }
}

#ifndef VLA_SKINNY_UNITS
#define VLA_SKINNY_UNITS 1536    // independent streams (waves) a decode GEMM is cut into, at least
#endif
// Number of partial planes (groups of 4 K slices) for an [N, K] weight matrix.
int skinny_ksplit(int N, int K) {
  const int NP = N / 64;
  int kg = (VLA_SKINNY_UNITS + 4 * NP - 1) / (4 * NP);
  if (kg < 1) kg = 1;
  if (kg > kMaxKSplit) kg = kMaxKSplit;
  while (kg > 1 && 4 * kg > K / 16) --kg;
  return kg;
}

void skinny_gemm(const f16* Afrag, const f16* Wp, float* part, int M, int N, int K, int kgroups, hipStream_t st) {
  const dim3 grid((N / 64) * kgroups), block(256);
  const int MT = (M + 31) / 32;
  const size_t smem = (size_t)2 * MT * 32 * 64 * sizeof(float);
#define VLA_SKINNY_CASE(MTV, DV)                                                                                  \
  case MTV: {                                                                                                     \
    auto kern = skinny_gemm_kernel<MTV, DV>;                                                                      \
    static bool attr_set = false;                                                                                 \
    if (!attr_set) {                                                                                              \
      (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);        \
      attr_set = true;                                                                                            \
    }                                                                                                             \
    hipLaunchKernelGGL(kern, grid, block, smem, st, Afrag, Wp, part, M, N, K, kgroups);                           \
  } break;
  switch (MT) {
    VLA_SKINNY_CASE(1, 8)
    VLA_SKINNY_CASE(2, 6)
    VLA_SKINNY_CASE(3, 4)
    VLA_SKINNY_CASE(4, 4)
    default: break;                                        // callers keep M <= 128
  }
#undef VLA_SKINNY_CASE
}

// ---- reduce + elementwise kernels ---------------------------------------------------------------------
__device__ __forceinline__ size_t frag_index(int m, int k, int K) {
  return ((size_t)(m >> 5) * (K >> 4) + (k >> 4)) * 512 + ((m & 31) + 32 * ((k >> 3) & 1)) * 8 + (k & 7);
}

__device__ __forceinline__ float block_sum_256d(float v, float* red) {
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// x[m,:] += sum_ks part[ks][m,:]; if gain: hn (fragment order) = f16(x * gain / rms(x)).
// Rows are handled in chunks: part holds rows 0..M-1 of the chunk, which are rows row0.. of x and hn.
__global__ __launch_bounds__(256) void reduce_resid_norm_kernel(const float* __restrict__ part, int ksplit, int M,
                                                                int d, float* __restrict__ x,
                                                                const float* __restrict__ gain, float eps,
                                                                f16* __restrict__ hn_frag, int row0) {
  __shared__ float red[4];
  const int m = blockIdx.x;
  float* row = x + (size_t)(row0 + m) * d;
  float ss = 0.f;
  for (int i = threadIdx.x * 4; i < d; i += 1024) {
    float4 v = *(const float4*)(row + i);
    float4 p[kMaxKSplit];
#pragma unroll
    for (int ks = 0; ks < kMaxKSplit; ++ks)            // all loads in flight first; summed in slice order
      p[ks] = ks < ksplit ? *(const float4*)(part + ((size_t)ks * M + m) * d + i) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int ks = 0; ks < kMaxKSplit; ++ks) {
      v.x += p[ks].x; v.y += p[ks].y; v.z += p[ks].z; v.w += p[ks].w;
    }
    *(float4*)(row + i) = v;
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  if (!gain) return;
  ss = block_sum_256d(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  for (int i = threadIdx.x * 4; i < d; i += 1024) {      // same mapping as above: a thread re-reads its own sums
    const float4 v = *(const float4*)(row + i);
    const float4 g = *(const float4*)(gain + i);
    typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
    f16x4 o;
    o[0] = from_f32<f16>(v.x * inv * g.x);
    o[1] = from_f32<f16>(v.y * inv * g.y);
    o[2] = from_f32<f16>(v.z * inv * g.z);
    o[3] = from_f32<f16>(v.w * inv * g.w);
    *(f16x4*)(hn_frag + frag_index(row0 + m, i, d)) = o;
  }
}

void reduce_resid_norm(const float* part, int ksplit, int M, int d, float* x, const float* gain, float eps,
                       f16* hn_frag, int row0, hipStream_t st) {
  hipLaunchKernelGGL(reduce_resid_norm_kernel, dim3(M), dim3(256), 0, st, part, ksplit, M, d, x, gain, eps, hn_frag,
                     row0);
}

// Plain RMSNorm of x rows into fragment order (first norm of a decode step).
__global__ __launch_bounds__(256) void rmsnorm_frag_kernel(const float* __restrict__ x, int d,
                                                           const float* __restrict__ gain, float eps,
                                                           f16* __restrict__ hn_frag) {
  __shared__ float red[4];
  const int m = blockIdx.x;
  const float* row = x + (size_t)m * d;
  float ss = 0.f;
  for (int i = threadIdx.x * 4; i < d; i += 1024) {
    const float4 v = *(const float4*)(row + i);
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ss = block_sum_256d(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  for (int i = threadIdx.x * 8; i < d; i += 2048) {
    f16x8 o;
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = from_f32<f16>(row[i + j] * inv * gain[i + j]);
    *(f16x8*)(hn_frag + frag_index(m, i, d)) = o;
  }
}
void rmsnorm_frag(const float* x, int M, int d, const float* gain, float eps, f16* hn_frag, hipStream_t st) {
  hipLaunchKernelGGL(rmsnorm_frag_kernel, dim3(M), dim3(256), 0, st, x, d, gain, eps, hn_frag);
}

// act (fragment order, [M, f]) = silu(gate) * up, gate/up summed over the K slices.  The fused
// gate-up columns are interleaved in blocks of 32: gate j at (j/32)*64 + j%32, up 32 further.
__global__ __launch_bounds__(256) void reduce_swiglu_kernel(const float* __restrict__ part, int ksplit, int M, int f,
                                                            f16* __restrict__ act_frag, int row0) {
  const int m = blockIdx.y;
  const int j0 = (blockIdx.x * 256 + threadIdx.x) * 8;      // 8 consecutive outputs (same 32-block)
  if (j0 >= f) return;
  const int col = (j0 >> 5) * 64 + (j0 & 31);
  float g[8] = {}, u[8] = {};
  for (int ks = 0; ks < ksplit; ++ks) {
    const float* p = part + ((size_t)ks * M + m) * (2 * (size_t)f) + col;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      g[j] += p[j];
      u[j] += p[32 + j];
    }
  }
  f16x8 o;
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = from_f32<f16>(g[j] / (1.0f + __expf(-g[j])) * u[j]);
  *(f16x8*)(act_frag + frag_index(row0 + m, j0, f)) = o;
}
void reduce_swiglu(const float* part, int ksplit, int M, int f, f16* act_frag, int row0, hipStream_t st) {
  hipLaunchKernelGGL(reduce_swiglu_kernel, dim3((f / 8 + 255) / 256, M), dim3(256), 0, st, part, ksplit, M, f, act_frag,
                     row0);
}

// q (row-major [M, d]) and the new K/V cache rows from the summed QKV partials, with RoPE.
__global__ __launch_bounds__(256) void reduce_qkv_rope_kernel(const float* __restrict__ part, int ksplit, int M,
                                                              RopeKv o, int row0) {
  const int m = blockIdx.x;
  const int d = o.d_model, hd = o.head_dim, half = hd >> 1;
  const int pos = o.tok_pos[row0 + m], slot = o.tok_seq[row0 + m];
  const size_t N = 3 * (size_t)d;
  for (int idx = threadIdx.x; idx < d / 2; idx += 256) {
    const int head = idx / half, i = idx - head * half;
    const int c0 = head * hd + i, c1 = c0 + half;
    float v[6] = {};
    for (int ks = 0; ks < ksplit; ++ks) {
      const float* p = part + ((size_t)ks * M + m) * N;
      v[0] += p[c0]; v[1] += p[c1]; v[2] += p[d + c0]; v[3] += p[d + c1]; v[4] += p[2 * d + c0]; v[5] += p[2 * d + c1];
    }
    const float cs = o.rope_cos[pos * half + i], sn = o.rope_sin[pos * half + i];
    f16* q = (f16*)o.q + (size_t)(row0 + m) * d;
    q[c0] = from_f32<f16>(v[0] * cs - v[1] * sn);
    q[c1] = from_f32<f16>(v[1] * cs + v[0] * sn);
    const size_t kv = (((size_t)slot * o.n_heads + head) * o.max_seq + pos) * hd;
    ((f16*)o.k_cache)[kv + i] = from_f32<f16>(v[2] * cs - v[3] * sn);
    ((f16*)o.k_cache)[kv + i + half] = from_f32<f16>(v[3] * cs + v[2] * sn);
    ((f16*)o.v_cache)[kv + i] = from_f32<f16>(v[4]);
    ((f16*)o.v_cache)[kv + i + half] = from_f32<f16>(v[5]);
  }
}
void reduce_qkv_rope(const float* part, int ksplit, int M, const RopeKv& o, int row0, hipStream_t st) {
  hipLaunchKernelGGL(reduce_qkv_rope_kernel, dim3(M), dim3(256), 0, st, part, ksplit, M, o, row0);
}

}  // namespace vla
