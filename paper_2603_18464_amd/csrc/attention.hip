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
    int n_items, int n_heads, int max_seq, bool out_frag) {
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
    if (out_frag) {   // [m/32][k/16][lane][8] fragment order with K = ldo (input of the decode GEMMs)
      const int m = tok, k = head * HD + i;
      out[((size_t)(m >> 5) * (ldo >> 4) + (k >> 4)) * 512 + ((m & 31) + 32 * ((k >> 3) & 1)) * 8 + (k & 7)] =
          from_f32<T>(acc * inv);
    } else {
      orow[i] = from_f32<T>(acc * inv);
    }
  }
}

// ---- prefill: causal flash attention on the matrix cores --------------------------------------------
// One workgroup = 4 waves = 128 consecutive query positions of one (sequence, head); each wave owns
// 32 queries.  Keys/values are walked in tiles of 64 positions staged in LDS.
//   S^T = K Q^T  : A operand = K rows (key-major, straight from the cache layout, XOR-swizzled 16-byte
//                  chunks in LDS), B operand = the wave's Q rows kept in registers.  In the 32x32
//                  accumulator layout every lane then owns ONE query (column l & 31) and 16 of the 32
//                  keys of a sub-tile, so the softmax statistics are per-lane scalars plus one exchange
//                  with lane ^ 32.
//   O^T += V^T P^T: B operand = P^T taken directly from the S^T accumulators (the contraction index
//                  may be permuted freely as long as both operands agree), A operand = V^T read from an
//                  LDS tile that was transposed while staging, with the key order inside each group of
//                  16 arranged so that a lane's 8 keys are contiguous.
// TWO (two-term mode): queries, keys and values each come as hi + lo terms (the low terms of the queries in half
// precision at column lo_off of the same rows, those of the cache as bytes, lo8 = bf8(16 * lo), in k_lo / v_lo
// with the cache's indexing; they are widened exactly to half precision while the tile is staged), the
// scores are K_hi Q_hi + K_lo Q_hi + K_hi Q_lo, the output sum takes V_hi + V_lo, and the output rows are written
// as [hi | lo] as well.  The staging tiles double, so one workgroup runs per compute unit instead of two.
template <int HD, bool TWO>
__global__ __launch_bounds__(256, 2) void flash_prefill_kernel(
    const f16* __restrict__ q, int ldq, const f16* __restrict__ k_cache, const f16* __restrict__ v_cache,
    const unsigned char* __restrict__ k_lo, const unsigned char* __restrict__ v_lo,
    const int32_t* __restrict__ cu_patch,
    const int32_t* __restrict__ cu_instr, const int32_t* __restrict__ slot_map, f16* __restrict__ out, int ldo,
    int n_heads, int max_seq, int lo_off, int out_lo8) {
  constexpr int KS = HD / 16;          // k-steps of the QK^T contraction
  constexpr int DT = HD / 32;          // 32-row tiles of O^T
  constexpr int KCH = HD / 8;          // 16-byte chunks per key row
  constexpr int VPITCH = 64 + 8;       // halves per V^T row (padding keeps b128 reads conflict free)
  constexpr int NP = TWO ? 2 : 1;      // planes: hi (and lo)
  __shared__ __attribute__((aligned(16))) f16 Ks[NP][64 * HD];
  __shared__ __attribute__((aligned(16))) f16 Vt[NP][HD * VPITCH];

  const int b = blockIdx.y, head = blockIdx.z;
  const int row0 = cu_patch[b] + cu_instr[b];
  const int S = cu_patch[b + 1] + cu_instr[b + 1] - row0;
  // Query tiles of 128 are aligned to the END of the sequence (the first tile is the short one): a tile needs the
  // keys up to its last query, so a prefix of 290 costs 1 + 3 + 5 key tiles instead of 2 + 4 + 5.
  const int nq = (S + 127) / 128;
  if ((int)blockIdx.x >= nq) return;
  const int q0 = S - 128 * (nq - (int)blockIdx.x);        // negative for a short first tile: those lanes are idle
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int qpos = q0 + wave * 32 + col;                 // this lane's query position (< S; idle if negative)
  const int qrow = row0 + max(qpos, 0);                   // clamped: idle lanes are never stored
  const int slot = slot_map ? slot_map[b] : b;
  const size_t blk = ((size_t)slot * n_heads + head) * max_seq * HD;
  const f16* kbase = k_cache + blk;
  const f16* vbase = v_cache + blk;
  const unsigned char* kbase8 = TWO ? k_lo + blk : nullptr;   // low terms of the cache: one byte per element
  const unsigned char* vbase8 = TWO ? v_lo + blk : nullptr;

  // Single-term: the wave's query fragments live in LDS (chunk c of query column `col` in slot c ^ (col & 7):
  // conflict-free 16-byte accesses); the registers they would occupy hold the prefetched next key / value tile
  // instead.  Two-term: the doubled key / value tiles take the LDS (two workgroups per compute unit must fit), so
  // the query fragments, high and low terms, stay in registers.
  __shared__ __attribute__((aligned(16))) f16 Qs[TWO ? 1 : 4][TWO ? 8 : 32 * HD];
  f16x8 qreg[TWO ? 2 : 1][TWO ? KS : 1];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const int ch = ks * 2 + half;
    if constexpr (TWO) {
      qreg[0][ks] = *(const f16x8*)(q + (size_t)qrow * ldq + head * HD + ch * 8);
      qreg[1][ks] = *(const f16x8*)(q + (size_t)qrow * ldq + lo_off + head * HD + ch * 8);
    } else {
      *(f16x8*)(Qs[wave] + col * HD + ((ch ^ (col & 7)) << 3)) =
          *(const f16x8*)(q + (size_t)qrow * ldq + head * HD + ch * 8);
    }
  }

  f32x16 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[dt][e] = 0.f;
  // Softmax statistics are kept in the base-2 domain: scores are scaled by log2(e) / sqrt(HD) once, and every
  // exponential is a bare exp2.  m_run is a reference point, not necessarily the running maximum: it is moved up
  // (and the accumulators rescaled) only when some query of the wave has found a score more than kLazy above it,
  // so most tiles skip the rescaling; probabilities relative to it stay below 2^kLazy, well inside half precision.
  float m_run = -INFINITY, l_run = 0.f;
  const float scale2 = rsqrtf((float)HD) * 1.44269504088896341f;
  constexpr float kLazy = 8.0f;

  const int kend = q0 + 128;                              // keys needed by this workgroup (<= S)
  const int wave_last = q0 + wave * 32 + 31;              // last query position of this wave
  // The next tile's keys and values are fetched into registers while the current tile is being consumed, so
  // the global-memory latency of a tile hides under the MFMAs and the softmax of the one before.
  constexpr int KI = 64 * KCH / 256, VI = 32 * KCH / 256;
  typedef __attribute__((ext_vector_type(2))) int i32x2;
  u32x4 kreg[KI];
  f16x8 vreg[VI][2];
  i32x2 kreg8[TWO ? KI : 1], vreg8[TWO ? VI : 1][2];       // the same items of the low-term planes, 8 bytes each
  auto fetch = [&](int k0) {                               // high terms of the tile at k0
#pragma unroll
    for (int i = 0; i < KI; ++i) {
      const int item = t + 256 * i;
      const int c = item % KCH, kk = item / KCH;
      const int kp = min(k0 + kk, S - 1);
      kreg[i] = *(const u32x4*)(kbase + (size_t)kp * HD + c * 8);
    }
#pragma unroll
    for (int i = 0; i < VI; ++i) {
      const int item = t + 256 * i;
      const int u = item & 31, c = item >> 5;
      const int ka = min(k0 + 2 * u, S - 1), kb = min(k0 + 2 * u + 1, S - 1);
      vreg[i][0] = *(const f16x8*)(vbase + (size_t)ka * HD + c * 8);
      vreg[i][1] = *(const f16x8*)(vbase + (size_t)kb * HD + c * 8);
    }
  };
  auto fetch8 = [&](int k0) {                              // low terms of the tile at k0
#pragma unroll
    for (int i = 0; i < KI; ++i) {
      const int item = t + 256 * i;
      const int c = item % KCH, kk = item / KCH;
      const int kp = min(k0 + kk, S - 1);
      kreg8[i] = *(const i32x2*)(kbase8 + (size_t)kp * HD + c * 8);
    }
#pragma unroll
    for (int i = 0; i < VI; ++i) {
      const int item = t + 256 * i;
      const int u = item & 31, c = item >> 5;
      const int ka = min(k0 + 2 * u, S - 1), kb = min(k0 + 2 * u + 1, S - 1);
      vreg8[i][0] = *(const i32x2*)(vbase8 + (size_t)ka * HD + c * 8);
      vreg8[i][1] = *(const i32x2*)(vbase8 + (size_t)kb * HD + c * 8);
    }
  };
  auto widen8 = [&](const i32x2& w) {                      // 8 low-term bytes -> half precision (exact)
    f16x8 h;
    h[0] = (f16)unpack_lo8(w[0], 0); h[1] = (f16)unpack_lo8(w[0], 1); h[2] = (f16)unpack_lo8(w[0], 2); h[3] = (f16)unpack_lo8(w[0], 3);
    h[4] = (f16)unpack_lo8(w[1], 0); h[5] = (f16)unpack_lo8(w[1], 1); h[6] = (f16)unpack_lo8(w[1], 2); h[7] = (f16)unpack_lo8(w[1], 3);
    return h;
  };
  fetch(0);
  for (int k0 = 0; k0 < kend; k0 += 64) {
    // Two-term: only the high terms are prefetched a tile ahead (the registers do not hold both); the low terms
    // are requested here, and the other workgroup on the compute unit covers their latency.
    if constexpr (TWO) fetch8(k0);
    __syncthreads();                                      // previous tile fully consumed
#pragma unroll
    for (int pl = 0; pl < NP; ++pl) {
      // K tile: 64 keys x KCH chunks, chunk c of key kk stored at slot c ^ (kk & 7) (low 3 bits)
#pragma unroll
      for (int i = 0; i < KI; ++i) {
        const int item = t + 256 * i;
        const int c = item % KCH, kk = item / KCH;
        u32x4 v = kreg[i];
        if constexpr (TWO) {
          if (pl == 1) v = __builtin_bit_cast(u32x4, widen8(kreg8[i]));
        }
        *(u32x4*)(Ks[pl] + kk * HD + ((c ^ (kk & 7)) << 3)) = v;
      }
      // V tile, transposed: Vt[dim][pos(key)], two keys per 32-bit store
#pragma unroll
      for (int i = 0; i < VI; ++i) {
        const int item = t + 256 * i;
        const int u = item & 31, c = item >> 5;
        const int g = (2 * u) & 15;                       // position of the key inside its group of 16
        const int pos = ((2 * u) & ~15) + ((g >> 2) & 1) * 8 + (g >> 3) * 4 + (g & 3);
        f16x8 va = vreg[i][0], vb = vreg[i][1];
        if constexpr (TWO) {
          if (pl == 1) {
            va = widen8(vreg8[i][0]);
            vb = widen8(vreg8[i][1]);
          }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
          f16x2 pr;
          pr[0] = va[j];
          pr[1] = vb[j];
          *(f16x2*)(Vt[pl] + (c * 8 + j) * VPITCH + pos) = pr;
        }
      }
    }
    __syncthreads();
    if (k0 + 64 < kend) fetch(k0 + 64);                   // uniform across the workgroup
    if (k0 > wave_last || wave_last < 0) continue;        // tile above this wave's diagonal, or no live query in the wave

    // S^T for the two 32-key sub-tiles
    f32x16 sacc[2];
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[st][e] = 0.f;
    // k-step outermost: one query fragment serves both key sub-tiles, and the two accumulator chains alternate
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      f16x8 qfr, qfl;
      if constexpr (TWO) {
        qfr = qreg[0][ks];
        qfl = qreg[1][ks];
      } else {
        qfr = *(const f16x8*)(Qs[wave] + col * HD + (((ks * 2 + half) ^ (col & 7)) << 3));
      }
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        const int kk = st * 32 + col;
        const int koff = kk * HD + (((ks * 2 + half) ^ (kk & 7)) << 3);
        const f16x8 kf = *(const f16x8*)(Ks[0] + koff);
        sacc[st] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qfr, sacc[st], 0, 0, 0);
        if constexpr (TWO) {
          const f16x8 kl = *(const f16x8*)(Ks[NP - 1] + koff);
          sacc[st] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kl, qfr, sacc[st], 0, 0, 0);
          sacc[st] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qfl, sacc[st], 0, 0, 0);
        }
      }
    }
    // scale, causal mask (only the tiles that reach past the wave's first query need one; a key position is below
    // S whenever it is at most the position of a live query), tile maximum
    float m_tile = -INFINITY;
    if (k0 + 63 > q0 + wave * 32) {
      // element (st, e) is key k0 + 4 * half + [st * 32 + 8 * (e >> 2) + (e & 3)]: visible iff [..] <= lim
      const int lim = qpos - k0 - 4 * half;
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float v = (st * 32 + 8 * (e >> 2) + (e & 3) <= lim) ? sacc[st][e] * scale2 : -INFINITY;
          sacc[st][e] = v;
          m_tile = fmaxf(m_tile, v);
        }
    } else {
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          sacc[st][e] *= scale2;
          m_tile = fmaxf(m_tile, sacc[st][e]);
        }
    }
    m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32, 64));
    if (__any(m_tile > m_run + kLazy)) {                    // (-inf + kLazy = -inf: true on the first live tile)
      const float m_new = fmaxf(m_run, m_tile);
      const float m_use = m_new == -INFINITY ? 0.f : m_new;  // fully masked so far: keep everything at zero
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);   // exp2(-inf) = 0 on the first live tile
      l_run *= alpha;
      m_run = m_new;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[dt][e] *= alpha;
    }
    const float m_ref = m_run == -INFINITY ? 0.f : m_run;
    float l_tile = 0.f;
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float p = __builtin_amdgcn_exp2f(sacc[st][e] - m_ref);
        sacc[st][e] = p;
        l_tile += p;
      }
    l_tile += __shfl_xor(l_tile, 32, 64);
    l_run += l_tile;
    // O^T += V^T P^T   (two-term mode: P too is split, P_hi V_hi + P_hi V_lo + P_lo V_hi)
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int ip = 0; ip < 2; ++ip) {
        f16x8 pf, pl8;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          pf[j] = (f16)sacc[st][8 * ip + j];
          if constexpr (TWO) pl8[j] = (f16)(sacc[st][8 * ip + j] - (float)pf[j]);
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const int voff = (dt * 32 + col) * VPITCH + st * 32 + ip * 16 + half * 8;
          const f16x8 vf = *(const f16x8*)(Vt[0] + voff);
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf, o[dt], 0, 0, 0);
          if constexpr (TWO) {
            const f16x8 vl = *(const f16x8*)(Vt[NP - 1] + voff);
            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vl, pf, o[dt], 0, 0, 0);
            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pl8, o[dt], 0, 0, 0);
          }
        }
      }
  }
  if (qpos >= 0) {
    const float inv = 1.0f / l_run;
    f16* orow = out + (size_t)(row0 + qpos) * ldo + head * HD;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
        f16x4 w, we;
        float e[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float v = o[dt][4 * i + r] * inv;
          w[r] = from_f32<f16>(v);
          e[r] = v - (float)w[r];
          we[r] = from_f32<f16>(e[r]);
        }
        *(f16x4*)(orow + dt * 32 + 8 * i + 4 * half) = w;
        if constexpr (TWO) {
          if (out_lo8)                                     // 8-bit low terms: bytes behind the row's lo_off high terms
            *(int*)((unsigned char*)(out + (size_t)(row0 + qpos) * ldo + lo_off) + head * HD + dt * 32 + 8 * i + 4 * half) =
                pack_lo8(e[0], e[1], e[2], e[3]);
          else
            *(f16x4*)(orow + lo_off + dt * 32 + 8 * i + 4 * half) = we;
        }
      }
  }
}

// k_lo / v_lo != nullptr selects the two-term kernel: q rows are [hi | lo] of pitch ldq with the low terms at
// column lo_off = d_model, and so are the output rows (pitch ldo), unless out_lo8 asks for 8-bit low terms (bytes
// behind the d_model high terms of each row).
void flash_prefill(const f16* q, int ldq, const f16* k_cache, const f16* v_cache, const unsigned char* k_lo,
                   const unsigned char* v_lo, const int32_t* cu_patch, const int32_t* cu_instr, const int32_t* slot_map,
                   f16* out, int ldo, bool out_lo8, int B, int max_len, int n_heads, int head_dim, int max_seq,
                   hipStream_t st) {
  const dim3 grid((max_len + 127) / 128, B, n_heads);
  const int lo_off = n_heads * head_dim;
#define VLA_FLASH(HDV, TWOV)                                                                                       \
  hipLaunchKernelGGL((flash_prefill_kernel<HDV, TWOV>), grid, dim3(256), 0, st, q, ldq, k_cache, v_cache, k_lo, v_lo, \
                     cu_patch, cu_instr, slot_map, out, ldo, n_heads, max_seq, lo_off, out_lo8 ? 1 : 0)
  if (k_lo) {
    if (head_dim == 128) VLA_FLASH(128, true);
    else VLA_FLASH(64, true);
  } else {
    if (head_dim == 128) VLA_FLASH(128, false);
    else VLA_FLASH(64, false);
  }
#undef VLA_FLASH
}

// ---- decode: one new query per (sequence, head) against the whole cache -------------------------------
// HBM-bound: the keys and values of a (slot, head) are one contiguous [position][HD] block each, and the
// kernel streams them once with 16-byte-per-lane loads (a wave instruction covers 64*16/(2*HD) whole
// rows).  One workgroup = 4 waves per (sequence, head); wave w takes every 4th group of rows.  A lane
// owns 8 head dimensions of one row at a time: scores are reduced across the HD/8 lanes of a row with
// shuffles, the probability-weighted values stay in 8 per-lane accumulators, and the partial softmax
// statistics and outputs of the waves are merged through LDS at the end.
//
// The query and the new key / value row of this (sequence, head) are not read from memory but formed here from
// the split-K partial sums of the QKV GEMM (summed in plane order, RoPE applied; the query stays in float32, the
// key / value row is rounded as the cache holds it); the new row is appended to the cache for the following steps
// and used from LDS in this one.
struct QkvPartials {
  const float* part;       // [ksplit][rows][3 * d_model]
  int ksplit, rows;
  const float* rope_cos;   // [max_seq, HD/2]
  const float* rope_sin;
};

// TWO (two-term mode): the cache holds every key / value as a half-precision high term plus a one-byte low term
// (k_lo / v_lo, same indexing, bf8(16 * lo)); both are streamed and added in float32; the output is written as hi
// and lo fragments (out_frag_lo).
template <int HD, bool TWO>
__global__ __launch_bounds__(256) void decode_attention_kernel(
    f16* __restrict__ k_cache, f16* __restrict__ v_cache,
    unsigned char* __restrict__ k_lo, unsigned char* __restrict__ v_lo, const int32_t* __restrict__ tok_seq,
    const int32_t* __restrict__ tok_pos,
    f16* __restrict__ out_frag, f16* __restrict__ out_frag_lo, int d_model, int n_heads, int max_seq,
    QkvPartials qp) {
  constexpr int LPR = HD / 8;            // lanes per row
  constexpr int RPI = 64 / LPR;          // rows per wave instruction
  __shared__ float s_m[4], s_l[4];
  __shared__ float s_o[4][HD];
  __shared__ __attribute__((aligned(16))) float s_q[HD], s_k[HD], s_v[HD];   // the new row, unrounded
  const int b = blockIdx.x, head = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane / LPR, c = lane % LPR;          // row inside the instruction, 8-dim chunk
  const int ctx = tok_pos[b] + 1;                      // >= 2 in a decode step: the prefix holds a position
  const int slot = tok_seq[b];
  const size_t blk = ((size_t)slot * n_heads + head) * max_seq * HD;
  f16* kb = k_cache + blk;
  f16* vb = v_cache + blk;
  unsigned char* kbl = TWO ? k_lo + blk : nullptr;     // low terms: one byte per element, bf8(16 * lo)
  unsigned char* vbl = TWO ? v_lo + blk : nullptr;
  const int last_global = ctx - 2;                     // last row that is read from the cache
  {
    constexpr int HALF = HD / 2;
    if (threadIdx.x < HALF) {
      const int i = threadIdx.x, c0 = head * HD + i, c1 = c0 + HALF, d = d_model, pos = ctx - 1;
      const size_t N = 3 * (size_t)d;
      float v[6] = {};
      for (int ks = 0; ks < qp.ksplit; ++ks) {
        const float* p = qp.part + ((size_t)ks * qp.rows + b) * N;
        v[0] += p[c0]; v[1] += p[c1]; v[2] += p[d + c0]; v[3] += p[d + c1]; v[4] += p[2 * d + c0]; v[5] += p[2 * d + c1];
      }
      const float cs = qp.rope_cos[pos * HALF + i], sn = qp.rope_sin[pos * HALF + i];
      float q0, q1, k0f, k1f;
      rope_pair(v[0], v[1], cs, sn, q0, q1);
      rope_pair(v[2], v[3], cs, sn, k0f, k1f);
      const f16 k0 = from_f32<f16>(k0f), k1 = from_f32<f16>(k1f);
      const f16 v0 = from_f32<f16>(v[4]), v1 = from_f32<f16>(v[5]);
      kb[(size_t)pos * HD + i] = k0; kb[(size_t)pos * HD + i + HALF] = k1;
      vb[(size_t)pos * HD + i] = v0; vb[(size_t)pos * HD + i + HALF] = v1;
      if constexpr (TWO) {
        const int ke = pack_lo8(k0f - (float)k0, k1f - (float)k1, v[4] - (float)v0, v[5] - (float)v1);
        kbl[(size_t)pos * HD + i] = (unsigned char)(ke & 0xff); kbl[(size_t)pos * HD + i + HALF] = (unsigned char)((ke >> 8) & 0xff);
        vbl[(size_t)pos * HD + i] = (unsigned char)((ke >> 16) & 0xff); vbl[(size_t)pos * HD + i + HALF] = (unsigned char)((ke >> 24) & 0xff);
        // this step uses exactly what later steps will read back: hi + lo
        s_q[i] = q0; s_q[i + HALF] = q1;
        s_k[i] = (float)k0 + unpack_lo8(ke, 0); s_k[i + HALF] = (float)k1 + unpack_lo8(ke, 1);
        s_v[i] = (float)v0 + unpack_lo8(ke, 2); s_v[i + HALF] = (float)v1 + unpack_lo8(ke, 3);
      } else {
        s_q[i] = q0; s_q[i + HALF] = q1;      // the query never leaves float32
        s_k[i] = (float)k0; s_k[i + HALF] = (float)k1; s_v[i] = (float)v0; s_v[i + HALF] = (float)v1;
      }
    }
    __syncthreads();
  }
  float qf[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) qf[j] = s_q[c * 8 + j];
  const float scale = rsqrtf((float)HD);

  // One pass with a running maximum per lane (row = (it*4 + wave)*RPI + sub): the key row and the value row of
  // an iteration are requested together, so twice as many bytes are in flight as with a score pass followed by
  // a value pass, and no scores have to be kept.
  float m_run = -INFINITY, lsum = 0.f;
  float acc[8] = {};
  const int n_it = (ctx + 4 * RPI - 1) / (4 * RPI);
  typedef __attribute__((ext_vector_type(2))) int i32x2;
  constexpr int U = 8;                     // iterations whose loads are issued together (16 rows of 16 bytes per lane)
  for (int it0 = 0; it0 < n_it; it0 += U) {
    f16x8 kv[U], vv[U];
    i32x2 kl[TWO ? U : 1], vl[TWO ? U : 1];               // low terms of the same rows: 8 bytes per lane
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = ((it0 + u) * 4 + wave) * RPI + sub;
      const size_t off = (size_t)min(row, last_global) * HD + c * 8;
      kv[u] = *(const f16x8*)(kb + off);
      vv[u] = *(const f16x8*)(vb + off);
      if constexpr (TWO) {
        kl[u] = *(const i32x2*)(kbl + off);
        vl[u] = *(const i32x2*)(vbl + off);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = ((it0 + u) * 4 + wave) * RPI + sub;
      float kf[8], vf[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        kf[j] = (float)kv[u][j];
        vf[j] = (float)vv[u][j];
        if constexpr (TWO) {
          kf[j] += unpack_lo8(kl[u][j >> 2], j & 3);
          vf[j] += unpack_lo8(vl[u][j >> 2], j & 3);
        }
      }
      if (row > last_global) {                               // the new row, from LDS
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          kf[j] = s_k[c * 8 + j];
          vf[j] = s_v[c * 8 + j];
        }
      }
      float s = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) s = fmaf(qf[j], kf[j], s);
#pragma unroll
      for (int o = LPR / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
      if (row < ctx) {                                      // uniform over the LPR lanes of a row
        s *= scale;
        const float m_new = fmaxf(m_run, s);
        const float alpha = __expf(m_run - m_new);          // exp(-inf) = 0 on the lane's first row
        const float p = __expf(s - m_new);
        lsum = lsum * alpha + p;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = fmaf(p, vf[j], acc[j] * alpha);
        m_run = m_new;
      }
    }
  }
  // bring the lanes of the wave to a common maximum, then add the row groups
  float mx = m_run;
#pragma unroll
  for (int o = 32; o >= LPR; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  {
    const float f = m_run == -INFINITY ? 0.f : __expf(m_run - mx);
    lsum *= f;
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] *= f;
  }
#pragma unroll
  for (int o = 32; o >= LPR; o >>= 1) {
    lsum += __shfl_xor(lsum, o, 64);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] += __shfl_xor(acc[j], o, 64);
  }
  if (sub == 0) {
#pragma unroll
    for (int j = 0; j < 8; ++j) s_o[wave][c * 8 + j] = acc[j];
    if (c == 0) { s_m[wave] = mx; s_l[wave] = lsum; }
  }
  __syncthreads();
  if (threadIdx.x < HD) {
    const int i = threadIdx.x;
    const float m = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
    float l = 0.f, o = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float f = s_m[w] == -INFINITY ? 0.f : __expf(s_m[w] - m);
      l += s_l[w] * f;
      o += s_o[w][i] * f;
    }
    const int k = head * HD + i;
    const size_t at = ((size_t)(b >> 5) * (d_model >> 4) + (k >> 4)) * 512 + ((b & 31) + 32 * ((k >> 3) & 1)) * 8 + (k & 7);
    const float r = o / l;
    const f16 r16 = from_f32<f16>(r);
    out_frag[at] = r16;
    if constexpr (TWO) out_frag_lo[at] = from_f32<f16>(r - (float)r16);
  }
}

// Row b of the step lives in cache slot tok_seq[b]; the query and the new cache row come from the QKV GEMM's partial
// sums part[ksplit][part_rows][3 * d_model].  k_lo != nullptr selects two-term mode.
void decode_attention_fused(const float* part, int ksplit, int part_rows, const float* rope_cos, const float* rope_sin,
                            f16* k_cache, f16* v_cache, unsigned char* k_lo, unsigned char* v_lo, const int32_t* tok_seq,
                            const int32_t* tok_pos, f16* out_frag, f16* out_frag_lo, int B, int d_model, int n_heads,
                            int head_dim, int max_seq, hipStream_t st) {
  const dim3 grid(B, n_heads);
  const QkvPartials qp{part, ksplit, part_rows, rope_cos, rope_sin};
#define VLA_DEC_ATT(HDV, TWOV)                                                                                     \
  hipLaunchKernelGGL((decode_attention_kernel<HDV, TWOV>), grid, dim3(256), 0, st, k_cache, v_cache,              \
                     k_lo, v_lo, tok_seq, tok_pos, out_frag, out_frag_lo, d_model, n_heads, max_seq, qp)
  if (k_lo) {
    if (head_dim == 128) VLA_DEC_ATT(128, true);
    else VLA_DEC_ATT(64, true);
  } else {
    if (head_dim == 128) VLA_DEC_ATT(128, false);
    else VLA_DEC_ATT(64, false);
  }
#undef VLA_DEC_ATT
}

template <class T>
void attention_rows(const T* q, int ldq, const T* k_cache, const T* v_cache, const int32_t* tok_seq,
                    const int32_t* tok_pos, T* out, int ldo, int n_tok, int n_heads, int head_dim, int max_seq,
                    bool out_frag, hipStream_t st) {
  const int n_items = n_tok * n_heads;
  const int blocks = (n_items + 3) / 4;
  const size_t smem = 4 * (size_t)(head_dim + max_seq) * sizeof(float);
#define VLA_ATTN_CASE(HD)                                                                                   \
  case HD:                                                                                                  \
    hipLaunchKernelGGL((attention_rows_kernel<T, HD>), dim3(blocks), dim3(256), smem, st, q, ldq, k_cache,  \
                       v_cache, tok_seq, tok_pos, out, ldo, n_items, n_heads, max_seq, out_frag);                     \
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
                                    float*, int, int, int, int, int, bool, hipStream_t);
}  // namespace vla
