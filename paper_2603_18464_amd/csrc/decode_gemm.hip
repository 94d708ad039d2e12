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

// TWO: two-term activations.  Af_lo holds the low terms in the same fragment order; every weight fragment is
// used for the hi and the lo activation fragments (weights are read once, the MFMA work doubles).
// Output rows: the M rows of this launch are rows row0 .. row0 + M - 1 of planes of plane_rows rows each.
template <int MT, int D, bool TWO>
__global__ __launch_bounds__(256, (MT <= 2 || !TWO) ? 2 : 1) void skinny_gemm_kernel(const f16* __restrict__ Af, const f16* __restrict__ Af_lo,
                                                          const f16* __restrict__ Wp, float* __restrict__ part, int M,
                                                          int N, int K, int kgroups, int plane_rows, int row0) {
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
  const f16* a0l = TWO ? Af_lo + lane * 8 : nullptr;

  // two arrays (one per 32-column block) rather than one: the compiler splits an array into scalars only up to a
  // bounded number of accesses, and an unsplit accumulator array would live in scratch memory
  f32x16 acc0[MT], acc1[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      acc0[i][e] = 0.f;
      acc1[i][e] = 0.f;
    }

  // Each wave walks its slice from a different starting point (rotated by its column pair).  The rows of
  // the packed matrix are a power-of-two number of bytes apart for K = 4096, so waves marching through k
  // in lockstep would all hit the same memory channels at the same time.
  const int len = kb_end - kb_begin;
  const int rot = (nbp * 5) % len;
  auto kb_of = [&](int i) {                                // i-th step of this wave, clamped to the slice
    const int j = min(i, len - 1) + rot;
    return (size_t)(kb_begin + (j >= len ? j - len : j));
  };
  constexpr int NA = TWO ? 2 * MT : MT;                    // activation fragments per k-step: hi (then lo)
  f16x8 wq[D][2], aq[D][NA];
  auto load_stage = [&](int s, size_t kb) {
    wq[s][0] = *(const f16x8*)(w0 + kb * 512);
    wq[s][1] = *(const f16x8*)(w1 + kb * 512);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      aq[s][mt] = *(const f16x8*)(a0 + ((size_t)mt * KB16 + kb) * 512);
      if constexpr (TWO) aq[s][MT + mt] = *(const f16x8*)(a0l + ((size_t)mt * KB16 + kb) * 512);
    }
  };
  auto mfma_stage = [&](int s) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      acc0[mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aq[s][mt], wq[s][0], acc0[mt], 0, 0, 0);
      acc1[mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aq[s][mt], wq[s][1], acc1[mt], 0, 0, 0);
      if constexpr (TWO) {
        acc0[mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aq[s][MT + mt], wq[s][0], acc0[mt], 0, 0, 0);
        acc1[mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aq[s][MT + mt], wq[s][1], acc1[mt], 0, 0, 0);
      }
    }
  };
#pragma unroll
  for (int s = 0; s < D; ++s) load_stage(s, kb_of(s));
  // Full groups of D k-steps: straight-line body (no branches, so the load counter is tracked exactly and
  // each MFMA waits only for its own stage); every consumed stage is refilled D steps ahead, clamped to the
  // last step of the slice.  The remaining steps (< D) sit in the first stages after the last group.
  const int n_full = len / D;
  for (int g = 0; g < n_full; ++g) {
    const int base = g * D;
#pragma unroll
    for (int s = 0; s < D; ++s) {
      mfma_stage(s);
      load_stage(s, kb_of(base + s + D));
      __builtin_amdgcn_sched_barrier(0);   // keep the refills in stage order, or the oldest stage's wait
                                           // degenerates into a wait for every outstanding load
    }
  }
  const int rem = len - n_full * D;
#pragma unroll
  for (int s = 0; s < D; ++s)
    if (s < rem) mfma_stage(s);
  // tree reduction over the four waves
  constexpr int REGS = MT * 32;
  auto put = [&](int slot) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        red[((size_t)slot * REGS + (mt * 2 + 0) * 16 + e) * 64 + lane] = acc0[mt][e];
        red[((size_t)slot * REGS + (mt * 2 + 1) * 16 + e) * 64 + lane] = acc1[mt][e];
      }
  };
  auto add = [&](int slot) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        acc0[mt][e] += red[((size_t)slot * REGS + (mt * 2 + 0) * 16 + e) * 64 + lane];
        acc1[mt][e] += red[((size_t)slot * REGS + (mt * 2 + 1) * 16 + e) * 64 + lane];
      }
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
  float* out = part + ((size_t)kg * plane_rows + row0) * N + nbp * 64 + c;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int blk = 0; blk < 4; ++blk)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = mt * 32 + 8 * blk + 4 * h + r;
        if (m < M) {
          out[(size_t)m * N] = acc0[mt][4 * blk + r] * (1.0f / kWeightScale);
          out[(size_t)m * N + 32] = acc1[mt][4 * blk + r] * (1.0f / kWeightScale);
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

// M <= kSkinnyMaxRows rows (fragment blocks Afrag / Afrag_lo start at the first of them); Afrag_lo != nullptr: two-term.
void skinny_gemm(const f16* Afrag, const f16* Afrag_lo, const f16* Wp, float* part, int M, int N, int K, int kgroups,
                 int plane_rows, int row0, hipStream_t st) {
  const dim3 grid((N / 64) * kgroups), block(256);
  const int MT = (M + 31) / 32;
  const size_t smem = (size_t)2 * MT * 32 * 64 * sizeof(float);
#define VLA_SKINNY_LAUNCH(MTV, DV, TWOV)                                                                          \
  {                                                                                                               \
    auto kern = skinny_gemm_kernel<MTV, DV, TWOV>;                                                                \
    static bool attr_set = false;                                                                                 \
    if (!attr_set) {                                                                                              \
      (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);        \
      attr_set = true;                                                                                            \
    }                                                                                                             \
    hipLaunchKernelGGL(kern, grid, block, smem, st, Afrag, Afrag_lo, Wp, part, M, N, K, kgroups, plane_rows, row0); \
  }
#define VLA_SKINNY_CASE(MTV, DV, DV2)                  \
  case MTV:                                            \
    if (Afrag_lo) VLA_SKINNY_LAUNCH(MTV, DV2, true)    \
    else VLA_SKINNY_LAUNCH(MTV, DV, false)             \
    break;
  switch (MT) {     // ring depth: as deep as the registers allow (weights 2 + activations MT or 2 MT fragments per stage)
    VLA_SKINNY_CASE(1, 8, 6)
    VLA_SKINNY_CASE(2, 6, 4)
    VLA_SKINNY_CASE(3, 4, 3)
    VLA_SKINNY_CASE(4, 3, 3)
    default: break;                                        // callers keep M <= kSkinnyMaxRows
  }
#undef VLA_SKINNY_CASE
#undef VLA_SKINNY_LAUNCH
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

// x[m,:] += sum_ks part[ks][m,:]; if gain: hn (fragment order) = f16(x * gain / rms(x)), and with hn_frag_lo the
// low terms f16(h - hi) as well.  Row m of the launch is row prow0 + m of each plane (plane_rows rows per plane) and
// row row0 + m of x and hn.
__global__ __launch_bounds__(256) void reduce_resid_norm_kernel(const float* __restrict__ part, int ksplit,
                                                                int plane_rows, int prow0, int d,
                                                                float* __restrict__ x, const float* __restrict__ gain,
                                                                float eps, f16* __restrict__ hn_frag,
                                                                f16* __restrict__ hn_frag_lo, int row0) {
  __shared__ float red[4];
  const int m = blockIdx.x;
  float* row = x + (size_t)(row0 + m) * d;
  float ss = 0.f;
  for (int i = threadIdx.x * 4; i < d; i += 1024) {
    float4 v = *(const float4*)(row + i);
    float4 p[kMaxKSplit];
#pragma unroll
    for (int ks = 0; ks < kMaxKSplit; ++ks)            // all loads in flight first; summed in slice order
      p[ks] = ks < ksplit ? *(const float4*)(part + ((size_t)ks * plane_rows + prow0 + m) * d + i)
                          : make_float4(0.f, 0.f, 0.f, 0.f);
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
    const float h[4] = {v.x * inv * g.x, v.y * inv * g.y, v.z * inv * g.z, v.w * inv * g.w};
    f16x4 o, oe;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      o[j] = from_f32<f16>(h[j]);
      oe[j] = from_f32<f16>(h[j] - (float)o[j]);
    }
    const size_t at = frag_index(row0 + m, i, d);
    *(f16x4*)(hn_frag + at) = o;
    if (hn_frag_lo) *(f16x4*)(hn_frag_lo + at) = oe;
  }
}

void reduce_resid_norm(const float* part, int ksplit, int plane_rows, int prow0, int M, int d, float* x,
                       const float* gain, float eps, f16* hn_frag, f16* hn_frag_lo, int row0, hipStream_t st) {
  hipLaunchKernelGGL(reduce_resid_norm_kernel, dim3(M), dim3(256), 0, st, part, ksplit, plane_rows, prow0, d, x, gain,
                     eps, hn_frag, hn_frag_lo, row0);
}

// Plain RMSNorm of x rows into fragment order (first norm of a decode step).
__global__ __launch_bounds__(256) void rmsnorm_frag_kernel(const float* __restrict__ x, int d,
                                                           const float* __restrict__ gain, float eps,
                                                           f16* __restrict__ hn_frag, f16* __restrict__ hn_frag_lo) {
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
    f16x8 o, oe;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float h = row[i + j] * inv * gain[i + j];
      o[j] = from_f32<f16>(h);
      oe[j] = from_f32<f16>(h - (float)o[j]);
    }
    const size_t at = frag_index(m, i, d);
    *(f16x8*)(hn_frag + at) = o;
    if (hn_frag_lo) *(f16x8*)(hn_frag_lo + at) = oe;
  }
}
void rmsnorm_frag(const float* x, int M, int d, const float* gain, float eps, f16* hn_frag, f16* hn_frag_lo,
                  hipStream_t st) {
  hipLaunchKernelGGL(rmsnorm_frag_kernel, dim3(M), dim3(256), 0, st, x, d, gain, eps, hn_frag, hn_frag_lo);
}

// act (fragment order, [M, f]) = silu(gate) * up, gate/up summed over the K slices.  The fused
// gate-up columns are interleaved in blocks of 32: gate j at (j/32)*64 + j%32, up 32 further.
__global__ __launch_bounds__(256) void reduce_swiglu_kernel(const float* __restrict__ part, int ksplit, int plane_rows,
                                                            int prow0, int f, f16* __restrict__ act_frag,
                                                            f16* __restrict__ act_frag_lo, int row0) {
  const int m = blockIdx.y;
  const int j0 = (blockIdx.x * 256 + threadIdx.x) * 8;      // 8 consecutive outputs (same 32-block)
  if (j0 >= f) return;
  const int col = (j0 >> 5) * 64 + (j0 & 31);
  float g[8] = {}, u[8] = {};
  for (int ks = 0; ks < ksplit; ++ks) {
    const float* p = part + ((size_t)ks * plane_rows + prow0 + m) * (2 * (size_t)f) + col;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      g[j] += p[j];
      u[j] += p[32 + j];
    }
  }
  f16x8 o, oe;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float a = g[j] / (1.0f + __expf(-g[j])) * u[j];
    o[j] = from_f32<f16>(a);
    oe[j] = from_f32<f16>(a - (float)o[j]);
  }
  const size_t at = frag_index(row0 + m, j0, f);
  *(f16x8*)(act_frag + at) = o;
  if (act_frag_lo) *(f16x8*)(act_frag_lo + at) = oe;
}
void reduce_swiglu(const float* part, int ksplit, int plane_rows, int prow0, int M, int f, f16* act_frag,
                   f16* act_frag_lo, int row0, hipStream_t st) {
  hipLaunchKernelGGL(reduce_swiglu_kernel, dim3((f / 8 + 255) / 256, M), dim3(256), 0, st, part, ksplit, plane_rows,
                     prow0, f, act_frag, act_frag_lo, row0);
}

}  // namespace vla
