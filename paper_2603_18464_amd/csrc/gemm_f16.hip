// Half-precision MFMA GEMM  C[M,N] = A[M,K] * W[N,K]^T  for gfx950, with the layer's elementwise
// work fused into the epilogue (residual add; SwiGLU; rotary embedding + KV-cache write).
//
// Operand layouts
//   A   row-major [M, lda] f16 (activations produced by this library).
//   Wp  weights (bf16 at the boundary, re-encoded exactly as f16 * kWeightScale) repacked once at
//       load time into MFMA fragment order: the 32x16 block
//       (rows n0..n0+31, k0..k0+15) is stored as 64 lanes x 8 halves = 1 KiB, lane l holding
//       row n0 + (l & 31), k = k0 + 8*(l >> 5) .. +7; blocks are ordered [n/32][k/16].  A wave
//       reads one block with a single fully coalesced 16-byte-per-lane load, from global memory or
//       from LDS, with no bank conflicts and no swizzle.
// The kernel keeps a BM x 64 slab of A (16-byte chunk c of row r sits in slot c ^ ((r >> 1) & 7), so
// that any 16 consecutive rows of one chunk column cover all 64 LDS banks) and a BN x 64 slab of Wp in
// LDS, double buffered, and each of the WGM x WGN waves owns a (BM/WGM) x (BN/WGN) accumulator tile made
// of 32x32x16 MFMAs.
#include "common.h"

namespace vla {

constexpr int BK = 64;

// ---- epilogues ------------------------------------------------------------------------------------
// Accumulator layout of v_mfma_f32_32x32x16_f16: lane l, register 4*blk + r holds
// C[row = 8*blk + 4*(l >> 5) + r][col = l & 31].

// Staged epilogues (large-tile kernel): a wave first writes a 32 x 128 float accumulator sub-tile to its
// private LDS region in row-major order (pitch kStagePitch floats: the two half-waves of a store hit
// disjoint banks), then reads it back as float4 row chunks, so that global memory sees 16-byte accesses
// that cover whole 128- to 512-byte row segments instead of scattered 2- and 4-byte ones.
constexpr int kStagePitch = 136;
constexpr int kStageFloats = 32 * kStagePitch;   // per wave

__device__ __forceinline__ void stage_tile(const f32x16 (&a)[4], float* tile, int lane) {
  const int h = lane >> 5, c = lane & 31;
#pragma unroll
  for (int nt = 0; nt < 4; ++nt)
#pragma unroll
    for (int e = 0; e < 16; ++e) tile[(8 * (e >> 2) + 4 * h + (e & 3)) * kStagePitch + nt * 32 + c] = a[nt][e];
}

struct EpiResid {
  float* x;
  int ldx;
  // rows m_base .. m_base+31, columns nb .. nb+127 of x += tile / kWeightScale
  __device__ __forceinline__ void consume(const float* tile, int m_base, int nb, int lane, int M) const {
    const int r0 = lane >> 5, c4 = (lane & 31) * 4;
    f32x4 v[16], old[16];
#pragma unroll
    for (int it = 0; it < 16; ++it) {
      const int r = it * 2 + r0;
      v[it] = *(const f32x4*)(tile + r * kStagePitch + c4);
      old[it] = *(const f32x4*)(x + (size_t)min(m_base + r, M - 1) * ldx + nb + c4);
    }
#pragma unroll
    for (int it = 0; it < 16; ++it) {
      const int m = m_base + it * 2 + r0;
      if (m < M) *(f32x4*)(x + (size_t)m * ldx + nb + c4) = old[it] + v[it] * (1.0f / kWeightScale);
    }
  }
  template <int MT, int NT>
  __device__ __forceinline__ void apply(f32x16 (&acc)[MT][NT], int mb, int nb, int lane, int M) const {
    const int h = lane >> 5, c = lane & 31;
    // Read-modify-write of the float32 residual stream.  All loads of a 32-row tile are issued before
    // its first store (a store followed by a load of the same array would otherwise serialise on the
    // memory latency); rows past M are read from row M-1 and not stored.
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      float old[16][NT];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = min(mb + mt * 32 + 8 * (e >> 2) + 4 * h + (e & 3), M - 1);
        const float* row = x + (size_t)m * ldx + nb + c;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) old[e][nt] = row[nt * 32];
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = mb + mt * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
        if (m < M) {
          float* row = x + (size_t)m * ldx + nb + c;
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) row[nt * 32] = old[e][nt] + acc[mt][nt][e] * (1.0f / kWeightScale);
        }
      }
    }
  }
};

// Fused gate/up weights are interleaved in blocks of 32 rows: [gate 0..31, up 0..31, gate 32..63, ...]
// so that a wave's even 32-column tiles are gates and the following odd tiles the matching ups.
// Split-K form (decode steps of large batches): the tile's partial sums over one K slice go, with the weight scale
// divided out, to plane `kz` of part[ksplit][plane_rows][N]; the reduce kernels of the decode path add the planes.
struct EpiPartial {
  float* part;          // plane 0; the kernel moves it to its slice's plane
  int plane_rows, row0, N;
  const f16* a_lo;      // low-term activation fragments (two-term operands), or nullptr
  __device__ __forceinline__ void consume(const float* tile, int m_base, int nb, int lane, int M) const {
    const int r0 = lane >> 5, c4 = (lane & 31) * 4;
#pragma unroll
    for (int it = 0; it < 16; ++it) {
      const int m = m_base + it * 2 + r0;
      const f32x4 v = *(const f32x4*)(tile + (it * 2 + r0) * kStagePitch + c4);
      if (m < M) *(f32x4*)(part + (size_t)(row0 + m) * N + nb + c4) = v * (1.0f / kWeightScale);
    }
  }
};

// silu(g) * u for accumulator values G = g * kWeightScale, U = u * kWeightScale, with the scale folded into the
// constants: (G * U / scale^2) / (1 + 2^(-G * log2(e) / scale)).  One form for both kernels (same bits).
__device__ __forceinline__ float swiglu_scaled(float G, float U) {
  constexpr float c1 = 1.44269504088896341f / kWeightScale, c2 = 1.0f / (kWeightScale * kWeightScale);
  return (G * U * c2) * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-(G * c1)));
}

struct EpiSwiglu {
  f16* act;
  int ld;
  int f;        // number of outputs per row
  int lo_mode;  // 0: single-term; 1: half-precision low terms at act[m][f + j]; 2: bytes at ((char*)&act[m][f])[j]
  // the 128 tile columns are [gate 32 | up 32 | gate 32 | up 32] -> 64 outputs per row
  __device__ __forceinline__ void consume(const float* tile, int m_base, int nb, int lane, int M) const {
    typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
    const int rs = lane >> 4, q = lane & 15, jb = q >> 3, c4 = (q & 7) * 4;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int r = it * 4 + rs, m = m_base + r;
      const f32x4 g = *(const f32x4*)(tile + r * kStagePitch + jb * 64 + c4);
      const f32x4 u = *(const f32x4*)(tile + r * kStagePitch + jb * 64 + 32 + c4);
      f16x4 o;
      float a[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        a[j] = swiglu_scaled(g[j], u[j]);
        o[j] = from_f32<f16>(a[j]);
      }
      if (m < M) {
        f16* row = act + (size_t)m * ld;
        *(f16x4*)(row + nb / 2 + jb * 32 + c4) = o;
        if (lo_mode != 0) {                  // (uniform) low terms only where the layer carries them
          float e[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) e[j] = a[j] - (float)o[j];
          if (lo_mode == 1) {
            f16x4 oe;
#pragma unroll
            for (int j = 0; j < 4; ++j) oe[j] = from_f32<f16>(e[j]);
            *(f16x4*)(row + f + nb / 2 + jb * 32 + c4) = oe;
          } else {
            *(int*)((unsigned char*)(row + f) + nb / 2 + jb * 32 + c4) = pack_lo8(e[0], e[1], e[2], e[3]);
          }
        }
      }
    }
  }
  template <int MT, int NT>
  __device__ __forceinline__ void apply(f32x16 (&acc)[MT][NT], int mb, int nb, int lane, int M) const {
    static_assert(NT % 2 == 0, "gate/up tiles come in pairs");
    const int h = lane >> 5, c = lane & 31;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int blk = 0; blk < 4; ++blk)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int m = mb + mt * 32 + 8 * blk + 4 * h + r;
          if (m < M) {
            f16* row = act + (size_t)m * ld + nb / 2 + c;
#pragma unroll
            for (int j = 0; j < NT / 2; ++j) {
              const float a = swiglu_scaled(acc[mt][2 * j][4 * blk + r], acc[mt][2 * j + 1][4 * blk + r]);
              const f16 a16 = from_f32<f16>(a);
              row[j * 32] = a16;
              if (lo_mode == 1) row[f + j * 32] = from_f32<f16>(a - (float)a16);
              if (lo_mode == 2)
                ((unsigned char*)(act + (size_t)m * ld + f))[nb / 2 + c + j * 32] =
                    (unsigned char)(pack_lo8(a - (float)a16, 0.f, 0.f, 0.f) & 0xff);
            }
          }
        }
  }
};

// Columns [0,d) are queries, [d,2d) keys, [2d,3d) values.  A wave tile covers whole heads, so the
// rotary partner (i, i + hd/2) of every column sits in the same lane, HD/64 tiles further on.
template <int HD>
struct EpiQkv {
  RopeKv o;
  // the 128 tile columns are 128/HD whole heads of one section (q, k or v)
  __device__ __forceinline__ void consume(const float* tile, int m_base, int nb, int lane, int M) const {
    typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
    constexpr int HALF = HD / 2, LPH = HD / 8;      // lanes per head: 16 lanes cover the 128/HD heads of a row
    const int rs = lane >> 4, q = lane & 15, hh = q / LPH, c4 = (q % LPH) * 4;
    const int d = o.d_model;
    const int sect = nb / d;
    const int head = (nb - sect * d) / HD + hh;
    // Positions, slots and rotary factors of all eight row groups are fetched up front (rows past M clamped), so
    // the two dependent global loads per row overlap instead of forming eight serial chains.
    int pos[8], slot[8];
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int m = min(m_base + it * 4 + rs, M - 1);
      pos[it] = o.tok_pos[m];
      slot[it] = o.tok_seq[m];
    }
    f32x4 cs[8], sn[8];
    if (sect < 2) {
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        cs[it] = *(const f32x4*)(o.rope_cos + (size_t)pos[it] * HALF + c4);
        sn[it] = *(const f32x4*)(o.rope_sin + (size_t)pos[it] * HALF + c4);
      }
    }
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int r = it * 4 + rs, m = m_base + r;
      f32x4 lo = *(const f32x4*)(tile + r * kStagePitch + hh * HD + c4) * (1.0f / kWeightScale);
      f32x4 hi = *(const f32x4*)(tile + r * kStagePitch + hh * HD + HALF + c4) * (1.0f / kWeightScale);
      f16* dst;
      f16* dst_lo = nullptr;                 // two-term mode: low terms of the queries (half precision, column d + ...)
      unsigned char* dst_lo8 = nullptr;      // ... and of the cached keys / values (one byte each)
      if (sect == 0) {
        dst = (f16*)o.q + (size_t)min(m, M - 1) * o.ldq + (size_t)head * HD;
        if (o.k_lo) dst_lo = dst + d;
      } else {
        const size_t at = (((size_t)slot[it] * o.n_heads + head) * o.max_seq + pos[it]) * HD;
        dst = (f16*)(sect == 1 ? o.k_cache : o.v_cache) + at;
        if (o.k_lo) dst_lo8 = (unsigned char*)(sect == 1 ? o.k_lo : o.v_lo) + at;
      }
      if (sect < 2) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float a, b;
          rope_pair(lo[j], hi[j], cs[it][j], sn[it][j], a, b);
          lo[j] = a;
          hi[j] = b;
        }
      }
      f16x4 l4, h4;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        l4[j] = from_f32<f16>(lo[j]);
        h4[j] = from_f32<f16>(hi[j]);
      }
      if (m < M) {
        *(f16x4*)(dst + c4) = l4;
        *(f16x4*)(dst + HALF + c4) = h4;
        if (o.k_lo) {                        // (uniform) low terms only in two-term layers
          float le[4], he[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            le[j] = lo[j] - (float)l4[j];
            he[j] = hi[j] - (float)h4[j];
          }
          if (dst_lo) {
            f16x4 l4e, h4e;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              l4e[j] = from_f32<f16>(le[j]);
              h4e[j] = from_f32<f16>(he[j]);
            }
            *(f16x4*)(dst_lo + c4) = l4e;
            *(f16x4*)(dst_lo + HALF + c4) = h4e;
          }
          if (dst_lo8) {
            *(int*)(dst_lo8 + c4) = pack_lo8(le[0], le[1], le[2], le[3]);
            *(int*)(dst_lo8 + HALF + c4) = pack_lo8(he[0], he[1], he[2], he[3]);
          }
        }
      }
    }
  }
  template <int MT, int NT>
  __device__ __forceinline__ void apply(f32x16 (&acc)[MT][NT], int mb, int nb, int lane, int M) const {
    constexpr int HT = HD / 32;              // 32-column tiles per head
    constexpr int HALF = HD / 2;
    static_assert(NT % HT == 0, "wave tile must cover whole heads");
    const int h = lane >> 5, c = lane & 31;
    const int d = o.d_model;
    const int sect = nb / d;                 // 0 q, 1 k, 2 v (a wave tile never straddles)
    const int col0 = nb - sect * d;          // first column inside the section
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int blk = 0; blk < 4; ++blk)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int m = mb + mt * 32 + 8 * blk + 4 * h + r;
          if (m >= M) continue;
          const int pos = o.tok_pos[m], slot = o.tok_seq[m];
          const int ai = 4 * blk + r;
          const float* cs_row = o.rope_cos + (size_t)pos * HALF;
          const float* sn_row = o.rope_sin + (size_t)pos * HALF;
#pragma unroll
          for (int hh = 0; hh < NT / HT; ++hh) {
            const int head = (col0 + hh * HD) / HD;
            f16* dst;
            f16* dst_lo = nullptr;
            unsigned char* dst_lo8 = nullptr;
            if (sect == 0) {
              dst = (f16*)o.q + (size_t)m * o.ldq + (size_t)head * HD;
              if (o.k_lo) dst_lo = dst + d;
            } else {
              const size_t at = (((size_t)slot * o.n_heads + head) * o.max_seq + pos) * HD;
              dst = (f16*)(sect == 1 ? o.k_cache : o.v_cache) + at;
              if (o.k_lo) dst_lo8 = (unsigned char*)(sect == 1 ? o.k_lo : o.v_lo) + at;
            }
#pragma unroll
            for (int ht = 0; ht < HT / 2; ++ht) {
              const int j = ht * 32 + c;     // index of the pair inside the head
              float lo = acc[mt][hh * HT + ht][ai] * (1.0f / kWeightScale);
              float hi = acc[mt][hh * HT + ht + HT / 2][ai] * (1.0f / kWeightScale);
              if (sect < 2) {
                float a, b;
                rope_pair(lo, hi, cs_row[j], sn_row[j], a, b);
                lo = a;
                hi = b;
              }
              const f16 l16 = from_f32<f16>(lo), h16 = from_f32<f16>(hi);
              dst[j] = l16;
              dst[j + HALF] = h16;
              if (dst_lo) {
                dst_lo[j] = from_f32<f16>(lo - (float)l16);
                dst_lo[j + HALF] = from_f32<f16>(hi - (float)h16);
              }
              if (dst_lo8) {
                dst_lo8[j] = (unsigned char)(pack_lo8(lo - (float)l16, 0.f, 0.f, 0.f) & 0xff);
                dst_lo8[j + HALF] = (unsigned char)(pack_lo8(hi - (float)h16, 0.f, 0.f, 0.f) & 0xff);
              }
            }
          }
        }
  }
};

// ---- 8-bit low terms --------------------------------------------------------------------------------------
// Two-term activations may carry their low term as one byte: lo8 = bf8(16 * (a - f16(a))) (1-5-2 format), stored
// behind the high terms of the same row, A row = [hi: Kw halves | lo8: Kw bytes].  The low-term product then runs
// on v_mfma_f32_32x32x64 in 8-bit formats (twice the rate of the half-precision instruction) against a second
// copy of the weights, W8 = fp8(w * 16) (1-4-3 format, saturating at +-448, i.e. |w| = 28), so that
// lo8 * W8 = 2^8 * lo * w lands in the same accumulator as hi * (w * 2^8).  The correction term only has to be good
// to a few percent (it is itself 2^-12 of the result), which three and two mantissa bits give.
// Layout: a 64-byte row slab of lo8 has the geometry of a 32-half slab of hi (64-byte rows), and W8 is packed so
// that its 64-k slab of a 32-row block is two 1 KiB pieces, lane (n, g) of piece j holding k = 32 j + 16 g .. + 15;
// a lane's operand is its 16 bytes of "k-step 0" followed by its 16 bytes of "k-step 1", for both operands.
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(8))) int i32x8;
__device__ __forceinline__ f32x16 mfma_lo8(const f16x8& a0, const f16x8& a1, const f16x8& b0, const f16x8& b1,
                                           const f32x16& c) {
#if defined(__HIP_DEVICE_COMPILE__)
  const i32x8 a = __builtin_shufflevector(__builtin_bit_cast(i32x4, a0), __builtin_bit_cast(i32x4, a1), 0, 1, 2, 3, 4, 5, 6, 7);
  const i32x8 b = __builtin_shufflevector(__builtin_bit_cast(i32x4, b0), __builtin_bit_cast(i32x4, b1), 0, 1, 2, 3, 4, 5, 6, 7);
  // A: bf8 (format 1), B: fp8 (format 0), no block scales
  return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 1, 0, 0, 0, 0, 0);
#else
  return c;
#endif
}

// ---- kernel -----------------------------------------------------------------------------------------
// LO8: the launch has 8-bit low-term slabs (W8 != nullptr); a template flag so that launches without them carry
// no trace of that pass and the two kinds of launch have names of their own in a profile.
template <int BM, int BN, int WGM, int WGN, class Epi, bool LO8>
__global__ __launch_bounds__(WGM* WGN * 64, 1) void gemm_f16_kernel(
    const f16* __restrict__ A, int lda, const f16* __restrict__ Wp, const f16* __restrict__ W8, int M, int N, int K,
    int Kw, int tiles_m, int tiles_n, Epi epi) {
  constexpr int NTHR = WGM * WGN * 64;
  constexpr int WTM = BM / WGM, WTN = BN / WGN, MT = WTM / 32, NT = WTN / 32;
  constexpr int A_ITERS = BM * 8 / NTHR;   // 16-byte chunks of the A slab per thread
  constexpr int W_ITERS = BN * 8 / NTHR;
  static_assert(BM * 8 % NTHR == 0 && BN * 8 % NTHR == 0, "slab must divide among threads");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  f16* As = (f16*)smem;                       // [2][BM*64]
  f16* Ws = As + 2 * BM * BK;                  // [2][BN*64]

  // XCD-aware tile order: consecutive workgroup ids land on different XCDs, so give each XCD a
  // contiguous run of tiles, walked in groups of GM row-tiles that share the same weight columns.
  const int nblk = tiles_m * tiles_n;
  const int per_xcd = gridDim.x >> 3;
  const int pid = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (pid >= nblk) return;
  constexpr int GM = 4;
  const int per_group = GM * tiles_n;
  const int grp = pid / per_group;
  const int first_m = grp * GM;
  const int gm = min(tiles_m - first_m, GM);
  const int in_grp = pid - grp * per_group;
  const int tm = first_m + in_grp % gm;
  const int tn = in_grp / gm;
  const int m0 = tm * BM, n0 = tn * BN;

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  // K == 2 * Kw: two-term A with half-precision low terms, the weight slabs wrap; K == 1.5 * Kw and W8: 8-bit low
  // terms (128 k per slab) against W8
  const int KB16 = Kw >> 4, KT = K / BK, KTw = Kw / BK;

  // Global -> register -> LDS staging.  Thread t moves 16-byte chunks: chunk (t & 7) of rows
  // (t >> 3) + i * NTHR/8 of the A slab (XOR-swizzled on the way into LDS), and the linear chunks
  // t + i * NTHR of the weight slab (fragment order needs no swizzle).
  const int a_c = t & 7, a_r = t >> 3;
  const f16* a_ptr[A_ITERS];
#pragma unroll
  for (int i = 0; i < A_ITERS; ++i)
    a_ptr[i] = A + (size_t)min(m0 + a_r + i * (NTHR / 8), M - 1) * lda + a_c * 8;
  const int a_dst = a_r * BK + ((a_c ^ ((a_r >> 1) & 7)) << 3);   // rows advance by multiples of 16: same swizzle
  const f16* w_ptr[W_ITERS];
#pragma unroll
  for (int i = 0; i < W_ITERS; ++i) {
    const int q = t + i * NTHR;
    w_ptr[i] = Wp + ((size_t)(n0 / 32 + (q >> 8)) * KB16) * 512 + (q & 255) * 8;
  }
  const f16* w8_ptr[W_ITERS];
#pragma unroll
  for (int i = 0; i < W_ITERS; ++i) {
    const int q = t + i * NTHR;
    w8_ptr[i] = W8 + ((size_t)(n0 / 32 + (q >> 8)) * KB16) * 256 + (q & 255) * 8;
  }

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  // fragment addresses inside a slab (elements)
  const int frow = wm * WTM + (lane & 31);
  const int fhalf = lane >> 5;
  int a_off[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) a_off[kk] = frow * BK + (((kk * 2 + fhalf) ^ ((frow >> 1) & 7)) << 3);
  const int w_off = wn * NT * 4 * 512 + lane * 8;

  u32x4 ra[A_ITERS], rw[W_ITERS];
#pragma unroll
  for (int i = 0; i < A_ITERS; ++i) ra[i] = *(const u32x4*)(a_ptr[i]);
#pragma unroll
  for (int i = 0; i < W_ITERS; ++i) rw[i] = *(const u32x4*)(w_ptr[i]);
#pragma unroll
  for (int i = 0; i < A_ITERS; ++i) *(u32x4*)(As + a_dst + i * (NTHR / 8) * BK) = ra[i];
#pragma unroll
  for (int i = 0; i < W_ITERS; ++i) *(u32x4*)(Ws + (t + i * NTHR) * 8) = rw[i];
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    // Prefetch the next slab into registers (the last iteration re-reads its own slab: harmless, and
    // it keeps the loop body one straight-line block that the scheduler can interleave freely).
    const int kn = min(kt + 1, KT - 1);
#pragma unroll
    for (int i = 0; i < A_ITERS; ++i) ra[i] = *(const u32x4*)(a_ptr[i] + kn * BK);
    const int knw = kn >= KTw ? kn - KTw : kn;
#pragma unroll
    for (int i = 0; i < W_ITERS; ++i)
      rw[i] = *(const u32x4*)((LO8 && kn >= KTw ? w8_ptr[i] : w_ptr[i]) + (size_t)knw * 4 * 512);
    __builtin_amdgcn_sched_barrier(0);   // keep the prefetch at the top: its latency hides under the MFMAs
    const f16* as = As + (kt & 1) * BM * BK;
    const f16* ws = Ws + (kt & 1) * BN * BK + w_off;
    if (LO8 && kt >= KTw) {              // a slab of 8-bit low terms: two 64-k products per accumulator tile
      f16x8 a4[4][MT], b4[4][NT];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) a4[kk][mt] = *(const f16x8*)(as + a_off[kk] + mt * 32 * BK);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) b4[kk][nt] = *(const f16x8*)(ws + (nt * 4 + kk) * 512);
      }
#pragma unroll
      for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            acc[mt][nt] = mfma_lo8(a4[2 * m][mt], a4[2 * m + 1][mt], b4[2 * m][nt], b4[2 * m + 1][nt], acc[mt][nt]);
      __builtin_amdgcn_sched_barrier(0);
      f16* asn = As + ((kt + 1) & 1) * BM * BK;
      f16* wsn = Ws + ((kt + 1) & 1) * BN * BK;
#pragma unroll
      for (int i = 0; i < A_ITERS; ++i) *(u32x4*)(asn + a_dst + i * (NTHR / 8) * BK) = ra[i];
#pragma unroll
      for (int i = 0; i < W_ITERS; ++i) *(u32x4*)(wsn + (t + i * NTHR) * 8) = rw[i];
      __syncthreads();
      continue;
    }
    f16x8 af[2][MT], bfr[2][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) af[0][mt] = *(const f16x8*)(as + a_off[0] + mt * 32 * BK);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) bfr[0][nt] = *(const f16x8*)(ws + nt * 4 * 512);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int cur = kk & 1, nxt = cur ^ 1;
      if (kk + 1 < 4) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) af[nxt][mt] = *(const f16x8*)(as + a_off[kk + 1] + mt * 32 * BK);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) bfr[nxt][nt] = *(const f16x8*)(ws + (nt * 4 + kk + 1) * 512);
      }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[cur][mt], bfr[cur][nt], acc[mt][nt], 0, 0, 0);
      // Scheduling hint: spread the LDS reads of the next k-step between the MFMAs of this one.
      if (kk + 1 < 4) {
#pragma unroll
        for (int i = 0; i < MT + NT; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, (MT * NT) / (MT + NT), 0);   // MFMA
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                       // DS read
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    f16* asn = As + ((kt + 1) & 1) * BM * BK;
    f16* wsn = Ws + ((kt + 1) & 1) * BN * BK;
#pragma unroll
    for (int i = 0; i < A_ITERS; ++i) *(u32x4*)(asn + a_dst + i * (NTHR / 8) * BK) = ra[i];
#pragma unroll
    for (int i = 0; i < W_ITERS; ++i) *(u32x4*)(wsn + (t + i * NTHR) * 8) = rw[i];
    __syncthreads();
  }
  epi.template apply<MT, NT>(acc, m0 + wm * WTM, n0 + wn * WTN, lane, M);
}

// ---- variant with direct global->LDS loads -----------------------------------------------------------
// Same tiling and LDS layout, but the slabs go from global memory straight into LDS
// (global_load_lds_dwordx4: lane l of a wave instruction deposits its 16 bytes at the wave-uniform
// LDS base + 16*l), so there is no register staging and no ds_write.  For the row-major A slab one
// instruction covers 8 rows x 128 bytes and the swizzle is applied on the source side: the lane that
// fills slot s of row r fetches chunk s ^ ((r >> 1) & 7).  The weight slab is already in fragment
// order, so it is a linear copy.  Per k-tile every wave first reads ALL its fragments of the current
// slab into registers, then issues the loads of the next slab into the other buffer, then runs its
// MFMAs; the loads have the whole MFMA phase to land and are waited for (vmcnt) only before the
// barrier that opens the next k-tile.
// 16 bytes per lane from global memory straight into LDS at lds_wave_base + 16 * lane.  The builtin only
// exists in the device pass; the host pass just needs the kernel's stub.
__device__ __forceinline__ void load_to_lds_16(const f16* src, f16* lds_wave_base) {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_global_load_lds(src, lds_wave_base, 16, 0, 0);
#else
  (void)src;
  (void)lds_wave_base;
#endif
}

// ---- 4-stage pipelined variant ------------------------------------------------------------------------
// 256x256 tiles, k-slabs of 32 (16 KiB of A + 16 KiB of W per stage, four stages = 128 KiB of LDS), loaded
// straight into LDS three slabs ahead of the MFMAs.  The compiler cannot tell the stages apart and would
// wait for ALL outstanding LDS loads before any LDS read, so the fragment reads are issued from inline
// assembly and the waits are explicit: vmcnt(2 * loads-per-slab) leaves the two newest slabs in flight,
// one barrier per slab publishes the landed slab and retires the oldest buffer, which is refilled at once.
// A slab layout: 64-byte rows, 16-byte chunk c of row r in slot c ^ ((r >> 2) & 3) (any 16 consecutive
// rows of a chunk column then cover all 64 banks); one load instruction covers 16 rows.
constexpr int PK = 32;                       // slab depth
constexpr int P_STAGES = 4;
constexpr int P_STAGE_HALVES = 256 * PK;     // per operand

// Issues the fragment reads of one slab (no wait).  The destination registers must not be touched
// until frags_arrived() has been executed on them.  Two wave tiles are supported: 64x128 and 128x128.
__device__ __forceinline__ void read_frags_asm(f16x8 (&af)[2][2], f16x8 (&bfr)[2][4], unsigned a0, unsigned a1,
                                               unsigned w) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile(
      "ds_read_b128 %0, %12\n\t"
      "ds_read_b128 %1, %12 offset:2048\n\t"
      "ds_read_b128 %4, %14\n\t"
      "ds_read_b128 %5, %14 offset:2048\n\t"
      "ds_read_b128 %6, %14 offset:4096\n\t"
      "ds_read_b128 %7, %14 offset:6144\n\t"
      "ds_read_b128 %2, %13\n\t"
      "ds_read_b128 %3, %13 offset:2048\n\t"
      "ds_read_b128 %8, %14 offset:1024\n\t"
      "ds_read_b128 %9, %14 offset:3072\n\t"
      "ds_read_b128 %10, %14 offset:5120\n\t"
      "ds_read_b128 %11, %14 offset:7168"
      : "=&v"(af[0][0]), "=&v"(af[0][1]), "=&v"(af[1][0]), "=&v"(af[1][1]), "=&v"(bfr[0][0]), "=&v"(bfr[0][1]),
        "=&v"(bfr[0][2]), "=&v"(bfr[0][3]), "=&v"(bfr[1][0]), "=&v"(bfr[1][1]), "=&v"(bfr[1][2]), "=&v"(bfr[1][3])
      : "v"(a0), "v"(a1), "v"(w)
      : "memory");
#endif
}
__device__ __forceinline__ void read_frags_asm(f16x8 (&af)[2][4], f16x8 (&bfr)[2][4], unsigned a0, unsigned a1,
                                               unsigned w) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile(
      "ds_read_b128 %0, %16\n\t"
      "ds_read_b128 %1, %16 offset:2048\n\t"
      "ds_read_b128 %8, %18\n\t"
      "ds_read_b128 %9, %18 offset:2048\n\t"
      "ds_read_b128 %2, %16 offset:4096\n\t"
      "ds_read_b128 %3, %16 offset:6144\n\t"
      "ds_read_b128 %10, %18 offset:4096\n\t"
      "ds_read_b128 %11, %18 offset:6144\n\t"
      "ds_read_b128 %4, %17\n\t"
      "ds_read_b128 %5, %17 offset:2048\n\t"
      "ds_read_b128 %12, %18 offset:1024\n\t"
      "ds_read_b128 %13, %18 offset:3072\n\t"
      "ds_read_b128 %6, %17 offset:4096\n\t"
      "ds_read_b128 %7, %17 offset:6144\n\t"
      "ds_read_b128 %14, %18 offset:5120\n\t"
      "ds_read_b128 %15, %18 offset:7168"
      : "=&v"(af[0][0]), "=&v"(af[0][1]), "=&v"(af[0][2]), "=&v"(af[0][3]), "=&v"(af[1][0]), "=&v"(af[1][1]),
        "=&v"(af[1][2]), "=&v"(af[1][3]), "=&v"(bfr[0][0]), "=&v"(bfr[0][1]), "=&v"(bfr[0][2]), "=&v"(bfr[0][3]),
        "=&v"(bfr[1][0]), "=&v"(bfr[1][1]), "=&v"(bfr[1][2]), "=&v"(bfr[1][3])
      : "v"(a0), "v"(a1), "v"(w)
      : "memory");
#endif
}

// Waits for every outstanding LDS read of this wave; the fragments are in/out operands so that nothing
// that uses them can be scheduled above the wait.
__device__ __forceinline__ void frags_arrived(f16x8 (&af)[2][2], f16x8 (&bfr)[2][4]) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(af[0][0]), "+v"(af[0][1]), "+v"(af[1][0]), "+v"(af[1][1]), "+v"(bfr[0][0]), "+v"(bfr[0][1]),
                 "+v"(bfr[0][2]), "+v"(bfr[0][3]), "+v"(bfr[1][0]), "+v"(bfr[1][1]), "+v"(bfr[1][2]), "+v"(bfr[1][3])
               :
               : "memory");
#endif
}
__device__ __forceinline__ void frags_arrived(f16x8 (&af)[2][4], f16x8 (&bfr)[2][4]) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(af[0][0]), "+v"(af[0][1]), "+v"(af[0][2]), "+v"(af[0][3]), "+v"(af[1][0]), "+v"(af[1][1]),
                 "+v"(af[1][2]), "+v"(af[1][3]), "+v"(bfr[0][0]), "+v"(bfr[0][1]), "+v"(bfr[0][2]), "+v"(bfr[0][3]),
                 "+v"(bfr[1][0]), "+v"(bfr[1][1]), "+v"(bfr[1][2]), "+v"(bfr[1][3])
               :
               : "memory");
#endif
}

// One fragment read with a compile-time byte offset (no wait; see frags_arrived).
template <int OFF>
__device__ __forceinline__ void read_frag_asm(f16x8& dst, unsigned addr) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF) : "memory");
#endif
}

// Waits until at most N LDS reads of this wave are outstanding (they complete in issue order) and ties the
// eight fragments of one k-step to the wait, so that nothing that uses them is scheduled above it.
template <int N>
__device__ __forceinline__ void frags_fence(f16x8 (&a)[4], f16x8 (&b)[4]) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_waitcnt lgkmcnt(%8)"
               : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3])
               : "n"(N)
               : "memory");
#endif
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
#endif
}

// SPLITK (with EpiPartial; one row of tiles, M <= 256): A is in the fragment order of the decode path
// ([m/32][k/16][lane][8], the low terms of two-term operands in a second buffer of the same order), `tiles_m` is
// the number of K slices, and workgroup (tile column tn, slice kz) accumulates slice kz of K only.
template <int WGM, int WGN, class Epi, bool LO8, bool SPLITK = false>
__global__ __launch_bounds__(WGM * WGN * 64, 1) void gemm_f16_pipe_kernel(const f16* __restrict__ A, int lda,
                                                                         const f16* __restrict__ Wp,
                                                                         const f16* __restrict__ W8, int M, int N,
                                                                         int K, int Kw, int tiles_m, int tiles_n,
                                                                         Epi epi_in) {
  constexpr int BM = 256, BN = 256, NW = WGM * WGN;
  constexpr int WTM = BM / WGM, WTN = BN / WGN, MT = WTM / 32, NT = WTN / 32;
  constexpr int A_INSTR = (BM / 16) / NW;      // 16 rows per load instruction -> 2 per wave
  constexpr int W_INSTR = (BN * PK * 2 / 1024) / NW;   // 2 per wave
  constexpr int LPS = A_INSTR + W_INSTR;       // loads per slab per wave
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  f16* As = (f16*)smem;                        // [4][256*32]
  f16* Ws = As + P_STAGES * P_STAGE_HALVES;    // [4][256*32]

  const int nblk = tiles_m * tiles_n;
  const int per_xcd = gridDim.x >> 3;
  const int pid = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (pid >= nblk) return;
  int tm, tn, kz = 0;
  if constexpr (SPLITK) {                      // consecutive workgroups of an XCD share a K slice (the A slabs)
    tm = 0;
    tn = pid % tiles_n;
    kz = pid / tiles_n;
  } else {
    constexpr int GM = 4;
    const int per_group = GM * tiles_n;
    const int grp = pid / per_group;
    const int first_m = grp * GM;
    const int gm = min(tiles_m - first_m, GM);
    const int in_grp = pid - grp * per_group;
    tm = first_m + in_grp % gm;
    tn = in_grp / gm;
  }
  const int m0 = tm * BM, n0 = tn * BN;
  Epi epi = epi_in;

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave / WGN, wn = wave % WGN;
  // K == 2 * Kw: two-term A with half-precision low terms, the weight slabs wrap; K == 1.5 * Kw and W8: 8-bit low
  // terms, whose slabs (64 k each, same bytes as a 32-k slab of halves) come after the KTw slabs of high terms
  const int KB16 = Kw >> 4;
  int KT = K / PK, KTw = Kw / PK;
  size_t slab0 = 0;                                      // first slab of this workgroup's K range
  if constexpr (SPLITK) {
    // slices in units of two slabs (64 k), so that every slice has an even number of slabs; K == 2 * Kw: the
    // slice of low-term slabs follows the slice of high-term slabs, against the same weight slabs
    const int U = Kw >> 6, u0 = (int)((long long)kz * U / tiles_m), u1 = (int)((long long)(kz + 1) * U / tiles_m);
    slab0 = 2 * (size_t)u0;
    KTw = 2 * (u1 - u0);
    KT = K > Kw ? 2 * KTw : KTw;
    epi.part += (size_t)kz * epi.plane_rows * epi.N;
  }

  const f16* a_src[A_INSTR];
  const f16* a_lo_src[A_INSTR];
#pragma unroll
  for (int i = 0; i < A_INSTR; ++i) {
    if constexpr (SPLITK) {
      const int j = wave * A_INSTR + i;                  // KiB of the slab: block row j/2 (clamped to the rows
      const int rb = min(j >> 1, (M - 1) >> 5);          // that exist), k-step j%2
      const size_t off = ((size_t)rb * KB16 + 2 * slab0 + (j & 1)) * 512 + lane * 8;
      a_src[i] = A + off;
      a_lo_src[i] = (epi.a_lo ? epi.a_lo : A) + off;
    } else {
      const int r = (wave * A_INSTR + i) * 16 + (lane >> 2);
      const int c = (lane & 3) ^ ((r >> 2) & 3);
      a_src[i] = A + (size_t)min(m0 + r, M - 1) * lda + c * 8;
      a_lo_src[i] = a_src[i];
    }
  }
  auto a_slab = [&](int i, int ks) {                     // source of the i-th activation load of slab ks
    if constexpr (SPLITK) return ks < KTw ? a_src[i] + (size_t)ks * 2 * 512 : a_lo_src[i] + (size_t)(ks - KTw) * 2 * 512;
    else return a_src[i] + (size_t)ks * PK;
  };
  const f16* w_src[W_INSTR];
#pragma unroll
  for (int i = 0; i < W_INSTR; ++i) {
    const int j = wave * W_INSTR + i;                    // KiB of the slab: block row j/2, k-step j%2
    w_src[i] = Wp + ((size_t)(n0 / 32 + (j >> 1)) * KB16 + 2 * slab0 + (j & 1)) * 512 + lane * 8;
  }
  const f16* w8_src[W_INSTR];
#pragma unroll
  for (int i = 0; i < W_INSTR; ++i) {
    const int j = wave * W_INSTR + i;
    w8_src[i] = W8 + (size_t)(n0 / 32 + (j >> 1)) * KB16 * 256 + (j & 1) * 512 + lane * 8;
  }
  auto w_slab = [&](int i, int ks) {                     // source of the i-th weight load of slab ks
    return ks < KTw ? w_src[i] + (size_t)ks * 2 * 512 : (LO8 ? w8_src[i] : w_src[i]) + (size_t)(ks - KTw) * 2 * 512;
  };
  auto issue = [&](int kt) {                             // slab kt (clamped) into buffer kt % 4
    const int buf = kt & (P_STAGES - 1);
    const int ks = min(kt, KT - 1);
    f16* as = As + buf * P_STAGE_HALVES + wave * A_INSTR * 512;
    f16* ws = Ws + buf * P_STAGE_HALVES + wave * W_INSTR * 512;
#pragma unroll
    for (int i = 0; i < A_INSTR; ++i) load_to_lds_16(a_slab(i, ks), as + i * 512);
#pragma unroll
    for (int i = 0; i < W_INSTR; ++i) load_to_lds_16(w_slab(i, ks), ws + i * 512);
  };

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  // LDS byte addresses of this lane's fragments inside buffer 0
  const unsigned lds0 = (unsigned)(size_t)((__attribute__((address_space(3))) unsigned char*)smem);
  const int frow = wm * WTM + (lane & 31);
  const int fhalf = lane >> 5;
  // (SPLITK: the A slab sits in LDS in fragment order like the weights: block row rb, k-step s at KiB 2 rb + s)
  const unsigned a_k0 = SPLITK ? lds0 + (unsigned)(wm * MT * 2) * 1024u + (unsigned)lane * 16u
                               : lds0 + 2u * (unsigned)(frow * PK + (((0 + fhalf) ^ ((frow >> 2) & 3)) << 3));
  const unsigned a_k1 = SPLITK ? a_k0 + 1024u
                               : lds0 + 2u * (unsigned)(frow * PK + (((2 + fhalf) ^ ((frow >> 2) & 3)) << 3));
  const unsigned w_b = lds0 + 2u * (unsigned)(P_STAGES * P_STAGE_HALVES + wn * NT * 2 * 512 + lane * 8);

  // Fragments are double buffered in registers: while the MFMAs of slab kt run, the reads of slab kt+1
  // are already in flight, so the LDS latency and the read burst after each barrier hide under MFMA work.
  f16x8 af[2][2][MT], bfr[2][2][NT];
  auto stage_off = [&](int kt) { return (unsigned)(kt & (P_STAGES - 1)) * (2u * P_STAGE_HALVES); };
  // One workgroup-wide slab step.  With two waves per SIMD (8 waves) the other wave's MFMAs cover this wave's
  // bursts of fragment reads and load issues; with one wave per SIMD (4 waves, 128x128 wave tile) every read and
  // every load is slotted between two MFMAs instead, so the matrix pipe never waits for the issue of a burst.
  auto issue_one = [&](int kt, int i) {      // i-th load instruction of slab kt (A first, then W)
    const int buf = kt & (P_STAGES - 1);
    const int ks = min(kt, KT - 1);
    if (i < A_INSTR)
      load_to_lds_16(a_slab(i, ks), As + buf * P_STAGE_HALVES + (wave * A_INSTR + i) * 512);
    else
      load_to_lds_16(w_slab(i - A_INSTR, ks), Ws + buf * P_STAGE_HALVES + (wave * W_INSTR + i - A_INSTR) * 512);
  };
  auto step = [&](int kt, int f) {           // f = kt & 1, passed as a constant by the unrolled caller
    wait_vmcnt<LPS>();                       // this wave's loads of slab kt+1 have landed (kt+2 may be in flight)
    __builtin_amdgcn_s_barrier();            // ... everyone's have; everyone holds slab kt in registers
    if constexpr (NW == 8) {
      // 16 MFMAs, and between them the 12 fragment reads of slab kt+1 and the 4 loads of slab kt+3, one each
      const unsigned so = stage_off(kt + 1);
      const unsigned ra0 = a_k0 + so, ra1 = a_k1 + so, rw = w_b + so;
#define VLA_MF(kk, mt, nt) \
  acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[f][kk][mt], bfr[f][kk][nt], acc[mt][nt], 0, 0, 0)
#define VLA_SB __builtin_amdgcn_sched_barrier(0)
      VLA_MF(0, 0, 0); read_frag_asm<0>(af[f ^ 1][0][0], ra0); VLA_SB;
      VLA_MF(0, 0, 1); read_frag_asm<0>(bfr[f ^ 1][0][0], rw); VLA_SB;
      VLA_MF(0, 0, 2); read_frag_asm<2048>(af[f ^ 1][0][1], ra0); VLA_SB;
      VLA_MF(0, 0, 3); read_frag_asm<2048>(bfr[f ^ 1][0][1], rw); VLA_SB;
      VLA_MF(0, 1, 0); read_frag_asm<4096>(bfr[f ^ 1][0][2], rw); VLA_SB;
      VLA_MF(0, 1, 1); read_frag_asm<6144>(bfr[f ^ 1][0][3], rw); VLA_SB;
      VLA_MF(0, 1, 2); read_frag_asm<0>(af[f ^ 1][1][0], ra1); VLA_SB;
      VLA_MF(0, 1, 3); read_frag_asm<2048>(af[f ^ 1][1][1], ra1); VLA_SB;
      VLA_MF(1, 0, 0); read_frag_asm<1024>(bfr[f ^ 1][1][0], rw); VLA_SB;
      VLA_MF(1, 0, 1); issue_one(kt + 3, 0); VLA_SB;
      VLA_MF(1, 0, 2); read_frag_asm<3072>(bfr[f ^ 1][1][1], rw); VLA_SB;
      VLA_MF(1, 0, 3); issue_one(kt + 3, 1); VLA_SB;
      VLA_MF(1, 1, 0); read_frag_asm<5120>(bfr[f ^ 1][1][2], rw); VLA_SB;
      VLA_MF(1, 1, 1); issue_one(kt + 3, 2); VLA_SB;
      VLA_MF(1, 1, 2); read_frag_asm<7168>(bfr[f ^ 1][1][3], rw); VLA_SB;
      VLA_MF(1, 1, 3); issue_one(kt + 3, 3); VLA_SB;
#undef VLA_MF
#undef VLA_SB
    } else {
      static_assert(NW == 8 || (MT == 4 && NT == 4 && LPS == 8), "interleaved schedule is written for 128x128 wave tiles");
      const unsigned so = stage_off(kt + 1);
      const unsigned ra0 = a_k0 + so, ra1 = a_k1 + so, rw = w_b + so;
#define VLA_MF(kk, mt, nt) \
  acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[f][kk][mt], bfr[f][kk][nt], acc[mt][nt], 0, 0, 0)
#define VLA_SB __builtin_amdgcn_sched_barrier(0)
      // Slots between the 32 MFMAs: a fragment read of slab kt+1 after every even one (first its k-step 0, then
      // its k-step 1), a load of slab kt+3 after every fourth.  The LDS thus sees one read per two MFMAs instead
      // of a burst, and the two waits below only ask for the eight reads that are needed next.
      VLA_MF(0, 0, 0); read_frag_asm<0>(af[f ^ 1][0][0], ra0); VLA_SB;
      VLA_MF(0, 0, 1); issue_one(kt + 3, 0); VLA_SB;
      VLA_MF(0, 0, 2); read_frag_asm<0>(bfr[f ^ 1][0][0], rw); VLA_SB;
      VLA_MF(0, 0, 3); VLA_SB;
      VLA_MF(0, 1, 0); read_frag_asm<2048>(af[f ^ 1][0][1], ra0); VLA_SB;
      VLA_MF(0, 1, 1); issue_one(kt + 3, 1); VLA_SB;
      VLA_MF(0, 1, 2); read_frag_asm<2048>(bfr[f ^ 1][0][1], rw); VLA_SB;
      VLA_MF(0, 1, 3); VLA_SB;
      VLA_MF(0, 2, 0); read_frag_asm<4096>(af[f ^ 1][0][2], ra0); VLA_SB;
      VLA_MF(0, 2, 1); issue_one(kt + 3, 2); VLA_SB;
      VLA_MF(0, 2, 2); read_frag_asm<4096>(bfr[f ^ 1][0][2], rw); VLA_SB;
      VLA_MF(0, 2, 3); VLA_SB;
      VLA_MF(0, 3, 0); read_frag_asm<6144>(af[f ^ 1][0][3], ra0); VLA_SB;
      VLA_MF(0, 3, 1); issue_one(kt + 3, 3); VLA_SB;
      VLA_MF(0, 3, 2); read_frag_asm<6144>(bfr[f ^ 1][0][3], rw); VLA_SB;
      VLA_MF(0, 3, 3); VLA_SB;
      // k-step 1 of slab kt was read during the second half of the previous step: eight newer reads may be pending
      frags_fence<8>(af[f][1], bfr[f][1]);
      VLA_SB;
      VLA_MF(1, 0, 0); read_frag_asm<0>(af[f ^ 1][1][0], ra1); VLA_SB;
      VLA_MF(1, 0, 1); issue_one(kt + 3, 4); VLA_SB;
      VLA_MF(1, 0, 2); read_frag_asm<1024>(bfr[f ^ 1][1][0], rw); VLA_SB;
      VLA_MF(1, 0, 3); VLA_SB;
      VLA_MF(1, 1, 0); read_frag_asm<2048>(af[f ^ 1][1][1], ra1); VLA_SB;
      VLA_MF(1, 1, 1); issue_one(kt + 3, 5); VLA_SB;
      VLA_MF(1, 1, 2); read_frag_asm<3072>(bfr[f ^ 1][1][1], rw); VLA_SB;
      VLA_MF(1, 1, 3); VLA_SB;
      VLA_MF(1, 2, 0); read_frag_asm<4096>(af[f ^ 1][1][2], ra1); VLA_SB;
      VLA_MF(1, 2, 1); issue_one(kt + 3, 6); VLA_SB;
      VLA_MF(1, 2, 2); read_frag_asm<5120>(bfr[f ^ 1][1][2], rw); VLA_SB;
      VLA_MF(1, 2, 3); VLA_SB;
      VLA_MF(1, 3, 0); read_frag_asm<6144>(af[f ^ 1][1][3], ra1); VLA_SB;
      VLA_MF(1, 3, 1); issue_one(kt + 3, 7); VLA_SB;
      VLA_MF(1, 3, 2); read_frag_asm<7168>(bfr[f ^ 1][1][3], rw); VLA_SB;
      VLA_MF(1, 3, 3); VLA_SB;
      // k-step 0 of slab kt+1 must be in registers before the next step; its k-step 1 may still be on its way
      frags_fence<8>(af[f ^ 1][0], bfr[f ^ 1][0]);
#undef VLA_MF
#undef VLA_SB
    }
    if constexpr (NW == 8) frags_arrived(af[f ^ 1], bfr[f ^ 1]);
  };
  // The same step for a slab of 8-bit low terms: one 64-k product per accumulator tile (as long as two of the
  // half-precision ones), operands = the lane's k-step 0 and k-step 1 fragments of the slab taken together.  All
  // fragment reads of slab kt+1 go into the first half of the step, so they have landed when it ends.
  auto step8 = [&](int kt, int f) {
    wait_vmcnt<LPS>();
    __builtin_amdgcn_s_barrier();
    frags_arrived(af[f], bfr[f]);            // both k-steps of slab kt are needed at once
    const unsigned so = stage_off(kt + 1);
    const unsigned ra0 = a_k0 + so, ra1 = a_k1 + so, rw = w_b + so;
#define VLA_MF8(mt, nt) acc[mt][nt] = mfma_lo8(af[f][0][mt], af[f][1][mt], bfr[f][0][nt], bfr[f][1][nt], acc[mt][nt])
#define VLA_SB __builtin_amdgcn_sched_barrier(0)
    if constexpr (NW == 8) {
      VLA_MF8(0, 0); read_frag_asm<0>(af[f ^ 1][0][0], ra0); read_frag_asm<0>(bfr[f ^ 1][0][0], rw); VLA_SB;
      VLA_MF8(0, 1); read_frag_asm<2048>(af[f ^ 1][0][1], ra0); read_frag_asm<2048>(bfr[f ^ 1][0][1], rw); VLA_SB;
      VLA_MF8(0, 2); read_frag_asm<4096>(bfr[f ^ 1][0][2], rw); read_frag_asm<6144>(bfr[f ^ 1][0][3], rw); VLA_SB;
      VLA_MF8(0, 3); read_frag_asm<0>(af[f ^ 1][1][0], ra1); read_frag_asm<2048>(af[f ^ 1][1][1], ra1); VLA_SB;
      VLA_MF8(1, 0); read_frag_asm<1024>(bfr[f ^ 1][1][0], rw); read_frag_asm<3072>(bfr[f ^ 1][1][1], rw); VLA_SB;
      VLA_MF8(1, 1); read_frag_asm<5120>(bfr[f ^ 1][1][2], rw); read_frag_asm<7168>(bfr[f ^ 1][1][3], rw); VLA_SB;
      VLA_MF8(1, 2); issue_one(kt + 3, 0); issue_one(kt + 3, 1); VLA_SB;
      VLA_MF8(1, 3); issue_one(kt + 3, 2); issue_one(kt + 3, 3); VLA_SB;
    } else {
      VLA_MF8(0, 0); read_frag_asm<0>(af[f ^ 1][0][0], ra0); read_frag_asm<0>(bfr[f ^ 1][0][0], rw); VLA_SB;
      VLA_MF8(0, 1); read_frag_asm<2048>(af[f ^ 1][0][1], ra0); read_frag_asm<2048>(bfr[f ^ 1][0][1], rw); VLA_SB;
      VLA_MF8(0, 2); read_frag_asm<4096>(af[f ^ 1][0][2], ra0); read_frag_asm<4096>(bfr[f ^ 1][0][2], rw); VLA_SB;
      VLA_MF8(0, 3); read_frag_asm<6144>(af[f ^ 1][0][3], ra0); read_frag_asm<6144>(bfr[f ^ 1][0][3], rw); VLA_SB;
      VLA_MF8(1, 0); read_frag_asm<0>(af[f ^ 1][1][0], ra1); read_frag_asm<1024>(bfr[f ^ 1][1][0], rw); VLA_SB;
      VLA_MF8(1, 1); read_frag_asm<2048>(af[f ^ 1][1][1], ra1); read_frag_asm<3072>(bfr[f ^ 1][1][1], rw); VLA_SB;
      VLA_MF8(1, 2); read_frag_asm<4096>(af[f ^ 1][1][2], ra1); read_frag_asm<5120>(bfr[f ^ 1][1][2], rw); VLA_SB;
      VLA_MF8(1, 3); read_frag_asm<6144>(af[f ^ 1][1][3], ra1); read_frag_asm<7168>(bfr[f ^ 1][1][3], rw); VLA_SB;
      VLA_MF8(2, 0); issue_one(kt + 3, 0); VLA_SB;
      VLA_MF8(2, 1); issue_one(kt + 3, 1); VLA_SB;
      VLA_MF8(2, 2); issue_one(kt + 3, 2); VLA_SB;
      VLA_MF8(2, 3); issue_one(kt + 3, 3); VLA_SB;
      VLA_MF8(3, 0); issue_one(kt + 3, 4); VLA_SB;
      VLA_MF8(3, 1); issue_one(kt + 3, 5); VLA_SB;
      VLA_MF8(3, 2); issue_one(kt + 3, 6); VLA_SB;
      VLA_MF8(3, 3); issue_one(kt + 3, 7); VLA_SB;
    }
#undef VLA_MF8
#undef VLA_SB
    frags_arrived(af[f ^ 1], bfr[f ^ 1]);
  };
  issue(0);
  issue(1);
  issue(2);
  wait_vmcnt<2 * LPS>();
  __builtin_amdgcn_s_barrier();
  read_frags_asm(af[0], bfr[0], a_k0, a_k1, w_b);
  frags_arrived(af[0], bfr[0]);
  const int KTh = LO8 ? KTw : KT;            // slabs of half-precision terms; the rest are 8-bit low terms
  for (int kt = 0; kt < KTh; kt += 2) {      // Kw is a multiple of 64: an even number of slabs
    step(kt, 0);
    step(kt + 1, 1);
  }
  if constexpr (LO8) {
    for (int kt = KTh; kt < KT; kt += 2) {   // Kw a multiple of 128 (the launcher checks): again an even number
      step8(kt, 0);
      step8(kt + 1, 1);
    }
  }
  if constexpr (NW == 4) {                   // the last step leaves eight fragment reads in flight: they must land
    frags_arrived(af[0], bfr[0]);            // before the registers they write are used for anything else
    frags_arrived(af[1], bfr[1]);
  }
  wait_vmcnt<0>();                           // the clamped tail loads still target this workgroup's LDS
  __syncthreads();                           // every wave is done with the slabs: LDS becomes epilogue staging
  float* tile = (float*)smem + wave * kStageFloats;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    stage_tile(acc[mt], tile, lane);
    epi.consume(tile, m0 + wm * WTM + mt * 32, n0 + wn * WTN, lane, M);
  }
}

template <int WGM, int WGN, class Epi, bool LO8>
static void launch_pipe(const GemmF16& g, const Epi& epi, hipStream_t st) {
  const int tiles_m = (g.M + 255) / 256, tiles_n = g.N / 256;
  const int nblk = tiles_m * tiles_n;
  const int grid = (nblk + 7) / 8 * 8;
  constexpr size_t slabs = 2 * (size_t)P_STAGES * P_STAGE_HALVES * sizeof(f16);
  constexpr size_t stage = (size_t)WGM * WGN * kStageFloats * sizeof(float);
  constexpr size_t smem = slabs > stage ? slabs : stage;
  auto kern = gemm_f16_pipe_kernel<WGM, WGN, Epi, LO8>;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(WGM * WGN * 64), smem, st, g.A, g.lda, g.Wp, g.W8, g.M, g.N, g.K, g.Kw,
                     tiles_m, tiles_n, epi);
}

// Decode GEMM of a large batch: partial sums of `ksplit` K slices, see EpiPartial and the SPLITK form of the kernel.
// Afrag / Afrag_lo: activation fragments of rows row0 .. row0 + M - 1 (their block row 0 = row row0, a multiple of 32).
bool splitk_gemm_fits(int M, int N, int K) { return M <= 256 && N % 256 == 0 && K % 64 == 0 && K >= 128; }
int splitk_ksplit(int N, int K) {
  int ks = 256 / (N / 256);                  // about one workgroup per compute unit
  if (ks > kMaxKSplit) ks = kMaxKSplit;
  while (ks > 1 && K / 64 < 4 * ks) --ks;    // at least 8 slabs per slice
  return ks < 1 ? 1 : ks;
}
void splitk_gemm(const f16* Afrag, const f16* Afrag_lo, const f16* Wp, float* part, int M, int N, int K, int ksplit,
                 int plane_rows, int row0, hipStream_t st) {
  const int tiles_n = N / 256, nblk = tiles_n * ksplit;
  const int grid = (nblk + 7) / 8 * 8;
  constexpr size_t slabs = 2 * (size_t)P_STAGES * P_STAGE_HALVES * sizeof(f16);
  constexpr size_t stage = (size_t)4 * kStageFloats * sizeof(float);
  constexpr size_t smem = slabs > stage ? slabs : stage;
  auto kern = gemm_f16_pipe_kernel<2, 2, EpiPartial, false, true>;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    attr_set = true;
  }
  const f16* no8 = nullptr;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), smem, st, Afrag, 0, Wp, no8, M, N, Afrag_lo ? 2 * K : K, K, ksplit,
                     tiles_n, EpiPartial{part, plane_rows, row0, N, Afrag_lo});
}

template <int BM, int BN, int WGM, int WGN, class Epi, bool LO8>
static void launch(const GemmF16& g, const Epi& epi, hipStream_t st) {
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = g.N / BN;
  const int nblk = tiles_m * tiles_n;
  const int grid = (nblk + 7) / 8 * 8;
  constexpr size_t smem = 2 * (size_t)(BM + BN) * BK * sizeof(f16);
  auto kern = gemm_f16_kernel<BM, BN, WGM, WGN, Epi, LO8>;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(WGM * WGN * 64), smem, st, g.A, g.lda, g.Wp, g.W8, g.M, g.N, g.K, g.Kw,
                     tiles_m, tiles_n, epi);
}

// Tile choice: big square tiles when there are enough rows to fill them, a 64-row tile for the
// decode-sized problems.  The QKV epilogue needs wave tiles that cover whole heads (128 columns).
// kWaves4: the 4-wave (128x128 wave tile) schedule reads a third less from LDS per MFMA and is the faster one
// for the residual and SwiGLU epilogues; the QKV epilogue measures marginally faster with 8 waves.
template <bool kWaves4, bool LO8, class Epi>
static void dispatch_lo(const GemmF16& g, const Epi& epi, hipStream_t st) {
  if (g.M > 128 && g.N % 256 == 0) {
    if (kWaves4) launch_pipe<2, 2, Epi, LO8>(g, epi, st);
    else launch_pipe<4, 2, Epi, LO8>(g, epi, st);
  } else if (g.N % 256 == 0) {
    launch<64, 256, 2, 2, Epi, LO8>(g, epi, st);
  } else {
    launch<64, 128, 2, 1, Epi, LO8>(g, epi, st);   // N multiple of 128
  }
}
template <bool kWaves4, class Epi>
static void dispatch(const GemmF16& g, const Epi& epi, hipStream_t st) {
  if (g.W8) dispatch_lo<kWaves4, true>(g, epi, st);
  else dispatch_lo<kWaves4, false>(g, epi, st);
}

void gemm_f16_resid(const GemmF16& g, float* x, int ldx, hipStream_t st) {
  dispatch<true>(g, EpiResid{x, ldx}, st);
}
void gemm_f16_swiglu(const GemmF16& g, f16* act, int ldact, int lo_mode, hipStream_t st) {
  dispatch<true>(g, EpiSwiglu{act, ldact, g.N / 2, lo_mode}, st);
}
void gemm_f16_qkv(const GemmF16& g, const RopeKv& o, hipStream_t st) {
  if (o.head_dim == 128) dispatch<false>(g, EpiQkv<128>{o}, st);
  else dispatch<false>(g, EpiQkv<64>{o}, st);
}

// ---- weight repacking -------------------------------------------------------------------------------
// Converts `rows` bf16 source rows [rows, K] to f16 * kWeightScale (exact: a power-of-two scale moves
// the exponent only, and f16 has more mantissa bits than bf16; values beyond +-255 saturate) and
// stores them in fragment order starting at packed row `row0`.  interleave_mode 0: packed row =
// row0 + r.  1 (gate) / 2 (up): rows go to the even / odd 32-row blocks of the fused gate-up matrix.
// One workgroup re-encodes 32 source rows x 512 k: 128-byte row segments are read coalesced, transposed through
// LDS, and each 1 KiB fragment block is written by one wave in one piece.
// range_flag (device int): bit 0 is set if a weight is too large for the re-encoding (|w| > 255) or not finite.
// (At the other end nothing is reported: 0 < |w| < 2^-25 falls between half-precision subnormals and is rounded
// with an absolute error below 2^-33, which is far below what any tolerance can see; random weights contain
// such values.)
// dst8 != nullptr: the same 32 x 64 spans also go, as fp8(w * 16) saturated at +-448, to the 8-bit copy
// [n/32][k/64][2 KiB]: piece j (1 KiB) of a span holds, for lane (n, g), the 16 bytes k = 32 j + 16 g .. + 15.
__global__ __launch_bounds__(256) void pack_weight_kernel(const bf16* __restrict__ src, int K,
                                                          f16* __restrict__ dst, unsigned char* __restrict__ dst8,
                                                          int row0, int mode, int* __restrict__ range_flag) {
  __shared__ u32x4 tile[32 * 8];
  const int r0 = blockIdx.x * 32;                       // first source row of this workgroup
  const int nb = mode == 0 ? (row0 + r0) >> 5 : (r0 >> 5) * 2 + (mode == 2 ? 1 : 0);
  const int t = threadIdx.x, rr = t >> 3, cc = t & 7;   // load role: row, 16-byte chunk of a 64-k span
  const int blk = t >> 6, lane = t & 63;                // store role: fragment block of the span, lane
  const int k_end = min(K, (int)(blockIdx.y + 1) * 512);
  int bad = 0;
  for (int k0 = blockIdx.y * 512; k0 < k_end; k0 += 64) {
    const bf16x8 v = *(const bf16x8*)(src + (size_t)(r0 + rr) * K + k0 + cc * 8);
    f16x8 o;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float w = (float)v[j], a = fabsf(w);
      if (!(a <= 255.0f)) bad |= 1;                     // also true for NaN
      o[j] = from_f32<f16>(w * kWeightScale);
    }
    __syncthreads();                                    // the previous span has been read out
    tile[rr * 8 + (cc ^ (rr & 7))] = __builtin_bit_cast(u32x4, o);
    __syncthreads();
    const int sr = lane & 31, sc = 2 * blk + (lane >> 5);
    *(u32x4*)(dst + ((size_t)nb * (K >> 4) + (k0 >> 4) + blk) * 512 + lane * 8) = tile[sr * 8 + (sc ^ (sr & 7))];
    if (dst8) {
#if defined(__HIP_DEVICE_COMPILE__)
      const int j8 = t >> 7, l8 = (t >> 1) & 63, h8 = t & 1;       // piece, lane, 8-byte half of the lane's 16 bytes
      const int n8 = l8 & 31, c8 = 4 * j8 + 2 * (l8 >> 5) + h8;    // row, 8-k chunk of the span
      const f16x8 w8 = __builtin_bit_cast(f16x8, tile[n8 * 8 + (c8 ^ (n8 & 7))]);
      float v8[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v8[j] = fminf(fmaxf((float)w8[j] * (kLo8Scale / kWeightScale), -448.0f), 448.0f);
      int p0 = __builtin_amdgcn_cvt_pk_fp8_f32(v8[0], v8[1], 0, false);
      p0 = __builtin_amdgcn_cvt_pk_fp8_f32(v8[2], v8[3], p0, true);
      int p1 = __builtin_amdgcn_cvt_pk_fp8_f32(v8[4], v8[5], 0, false);
      p1 = __builtin_amdgcn_cvt_pk_fp8_f32(v8[6], v8[7], p1, true);
      int* o8 = (int*)(dst8 + ((size_t)nb * (K >> 6) + (k0 >> 6)) * 2048 + j8 * 1024 + l8 * 16 + h8 * 8);
      o8[0] = p0;
      o8[1] = p1;
#endif
    }
  }
  if (bad) atomicOr(range_flag, bad);
}

void pack_weight_f16(const bf16* src, int rows, int K, f16* dst, unsigned char* dst8, int row0, int interleave_mode,
                     int* range_flag, hipStream_t st) {
  // rows, row0 multiples of 32 and K a multiple of 64: guaranteed by the configuration checks
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)(rows / 32), (unsigned)((K + 511) / 512)), dim3(256), 0, st,
                     src, K, dst, dst8, row0, interleave_mode, range_flag);
}

}  // namespace vla
