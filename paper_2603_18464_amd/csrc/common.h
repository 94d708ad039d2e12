// Shared device helpers and the host-side launcher declarations of the VLA policy library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vla {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef _Float16 f16;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kWave = 64;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
__device__ __forceinline__ float to_f32(f16 v) { return (float)v; }
template <class T> __device__ __forceinline__ T from_f32(float v);
// float -> half, IEEE round to nearest even: a value beyond the half-precision range becomes an infinity and a
// NaN stays a NaN, so an overflow or a non-finite input reaches the logits and the log-probs as NaN instead of
// being clamped to something plausible.
template <> __device__ __forceinline__ f16 from_f32<f16>(float v) { return (f16)v; }
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ---- kernel families timed by the profiling hooks ----------------------------------------------
enum Family {
  FAM_GEMM_QKV_PREFILL = 0,
  FAM_GEMM_O_PREFILL,
  FAM_GEMM_GATEUP_PREFILL,
  FAM_GEMM_DOWN_PREFILL,
  FAM_ATTN_PREFILL,
  FAM_GEMM_QKV_DECODE,
  FAM_GEMM_O_DECODE,
  FAM_GEMM_GATEUP_DECODE,
  FAM_GEMM_DOWN_DECODE,
  FAM_ATTN_DECODE,
  FAM_NORM,
  FAM_HEAD,
  FAM_MISC,
  FAM_TAIL,      // last prefill layer restricted to the rows that feed the head
  FAM_GEMM_QKV_TWO_PREFILL,      // the prefill GEMMs of two-term layers (with their low-term pass), same order
  FAM_GEMM_O_TWO_PREFILL,
  FAM_GEMM_GATEUP_TWO_PREFILL,
  FAM_GEMM_DOWN_TWO_PREFILL,
  FAM_COUNT
};

// ---- launcher arguments ---------------------------------------------------------------------------
struct RopeKv {
  void* q;               // [T, ldq] storage dtype, rotated queries (two-term mode: columns [d_model, 2 d_model) hold the low terms)
  void* k_cache;         // layer base: [slot][head][position][head_dim]
  void* v_cache;
  void* k_lo;            // two-term mode: low terms of the cached keys / values, same indexing, one byte per element
  void* v_lo;            //   (bf8(16 * lo)); nullptr otherwise
  int ldq;               // row pitch of q in elements
  const int32_t* tok_seq;   // [T] slot of each packed token
  const int32_t* tok_pos;   // [T] position of each packed token inside its sequence
  const float* rope_cos;    // [max_seq, head_dim/2]
  const float* rope_sin;
  int n_heads, head_dim, max_seq, d_model;   // max_seq: positions per (slot, head) block of the cache (its pitch)
};

// The 16-bit path keeps weights as bfloat16 at the boundary but feeds the matrix cores in half
// precision: bf16 -> f16 is exact once the weights are scaled by a power of two (kWeightScale keeps
// |w| up to 255 finite and everything above 2^-25 exact), activations rounded to f16 carry 8x less
// rounding error than bf16 at the same MFMA rate, and the scale is divided out in the epilogue.
constexpr float kWeightScale = 256.0f;
constexpr int kMaxKSplit = 4;   // most partial planes (groups of 4 K slices) a decode GEMM writes

// Two-term activations: a value a is carried as hi = f16(a) and lo = f16(a - hi) (together about 22 significant
// bits).  Row-major operands keep them side by side, A = [hi | lo] with K = 2 * Kw columns; since the weights
// are exact, A * W^T = hi * W^T + lo * W^T is one contraction over 2 * Kw in which the weight index wraps.
struct GemmF16 {
  const f16* A;    // [M, K] row-major activations
  int lda;
  const f16* Wp;   // [N, Kw] weights * kWeightScale in MFMA fragment order (see pack_weight_f16)
  int M, N, K;     // K = Kw (single-term A), 2 * Kw (two-term A, half-precision low terms) or, with W8, 1.5 * Kw
  int Kw;          //   (two-term A whose low terms are bytes: row = [hi: Kw halves | lo8: Kw bytes]; Kw % 128 == 0)
  const f16* W8;   // 8-bit copy of the weights for 8-bit low terms (see gemm_f16.hip), or nullptr
};
// 8-bit low terms (see gemm_f16.hip): lo8 = bf8(16 * (a - f16(a))), four at a time.
constexpr float kLo8Scale = 16.0f;
__device__ __forceinline__ int pack_lo8(float e0, float e1, float e2, float e3) {
#if defined(__HIP_DEVICE_COMPILE__)
  int p = __builtin_amdgcn_cvt_pk_bf8_f32(e0 * kLo8Scale, e1 * kLo8Scale, 0, false);
  return __builtin_amdgcn_cvt_pk_bf8_f32(e2 * kLo8Scale, e3 * kLo8Scale, p, true);
#else
  return 0;
#endif
}
__device__ __forceinline__ float unpack_lo8(int word, int byte) {   // byte must be a compile-time constant 0..3
#if defined(__HIP_DEVICE_COMPILE__)
  float v;
  switch (byte) {
    case 0: v = __builtin_amdgcn_cvt_f32_bf8(word, 0); break;
    case 1: v = __builtin_amdgcn_cvt_f32_bf8(word, 1); break;
    case 2: v = __builtin_amdgcn_cvt_f32_bf8(word, 2); break;
    default: v = __builtin_amdgcn_cvt_f32_bf8(word, 3); break;
  }
  return v * (1.0f / kLo8Scale);
#else
  return 0.f;
#endif
}

// Rotation of one pair by (cos, sin), written with explicit roundings: every kernel that applies it (the two
// epilogue forms of the QKV GEMM, the decode step) then produces the same float32 bits, which two-term outputs
// make visible.
__device__ __forceinline__ void rope_pair(float lo, float hi, float cs, float sn, float& a, float& b) {
  a = __fmaf_rn(lo, cs, -__fmul_rn(hi, sn));
  b = __fmaf_rn(hi, cs, __fmul_rn(lo, sn));
}

// C = A * W^T with fused epilogues (f16 MFMA, fp32 accumulation).
void gemm_f16_resid(const GemmF16& g, float* x, int ldx, hipStream_t st);           // x += C
// silu(gate)*up; lo_mode 1: also half-precision low terms at column f + j; 2: 8-bit low terms, bytes behind the f halves
void gemm_f16_swiglu(const GemmF16& g, f16* act, int ldact, int lo_mode, hipStream_t st);
void gemm_f16_qkv(const GemmF16& g, const RopeKv& o, hipStream_t st);               // RoPE + cache
// range_flag: device int, bits are OR-ed in when a weight cannot be re-encoded exactly (see pack_weight_kernel);
// dst8 != nullptr: also the 8-bit copy fp8(w * 16) for 8-bit low terms (K % 64 == 0)
void pack_weight_f16(const bf16* src, int rows, int K, f16* dst, unsigned char* dst8, int row0, int interleave_mode,
                     int* range_flag, hipStream_t st);

// fp32 path (plain, unfused).
void gemm_f32(const float* A, int lda, const float* W, float* C, int M, int N, int K, hipStream_t st);
void rope_kv_f32(const float* qkv, int T, const RopeKv& o, hipStream_t st);
void resid_add_f32(float* x, const float* c, size_t n, hipStream_t st);
void swiglu_f32(const float* gu, float* act, int T, int f, hipStream_t st);

// Row-wise kernels.
template <class T>
void rmsnorm(const float* x, const T* /*unused tag*/, const float* gain, T* out, int rows, int d,
             float eps, const int32_t* row_index, int lo_mode /* 0: rows of d; 1: [hi | lo] of 2 d; 2: [hi | lo8] of 1.5 d */,
             hipStream_t st);
template <class T>
void assemble_prefix(const T* patch_emb, const int32_t* instr_ids, const T* embed,
                     const int32_t* tok_src, float* x, int T_tokens, int d, int vocab, hipStream_t st);
template <class T>
void embed_tokens(const int32_t* ids, const T* embed, float* x, int B, int d, int vocab, hipStream_t st);

// Attention: one query row per (token, head) against the cache.
template <class T>
void attention_rows(const T* q, int ldq, const T* k_cache, const T* v_cache, const int32_t* tok_seq,
                    const int32_t* tok_pos, T* out, int ldo, int n_tok, int n_heads, int head_dim,
                    int max_seq, bool out_frag, hipStream_t st);

// Prefill attention for the 16-bit path: causal flash attention over whole prefixes (MFMA).
// cu_patch / cu_instr are the device copies of the cumulative offsets; max_len = longest prefix; slot_map
// (device, [B], or nullptr for the identity) gives the cache slot of each sequence of the call.
// k_lo / v_lo (low terms of the cache) != nullptr: two-term mode, q rows are [hi | lo] with the low terms at column
// d_model, and so are the output rows, or (out_lo8) [hi | 8-bit low terms].
void flash_prefill(const f16* q, int ldq, const f16* k_cache, const f16* v_cache, const unsigned char* k_lo,
                   const unsigned char* v_lo, const int32_t* cu_patch, const int32_t* cu_instr, const int32_t* slot_map,
                   f16* out, int ldo, bool out_lo8, int B, int max_len, int n_heads, int head_dim, int max_seq,
                   hipStream_t st);

// Decode-step GEMMs (M <= 128): weight-streaming split-K kernel writing partial sums, and the kernels
// that add the partials in a fixed order and apply the elementwise step that follows each GEMM.
// Activations named *_frag are [M, K] in MFMA fragment order: [m/32][k/16][lane][8].
int skinny_ksplit(int N, int K);
constexpr int kSkinnyMaxRows = 128;   // most rows of one weight-streaming GEMM launch
// Two-term mode: *_lo arguments hold the low terms f16(a - f16(a)) in the same fragment order (nullptr: single-term).
// The M rows of a launch are rows prow0 .. prow0 + M - 1 of partial planes of plane_rows rows each.
void skinny_gemm(const f16* Afrag, const f16* Afrag_lo, const f16* Wp, float* part, int M, int N, int K, int ksplit,
                 int plane_rows, int prow0, hipStream_t st);
// The same product for up to 256 rows on the 256 x 256 tiled kernel, split over `ksplit` K slices (one partial plane
// each): activations go through LDS once per workgroup instead of once per wave, which is what a large batch needs
// to stream every weight once at full rate.  Needs N % 256 == 0 and K % 64 == 0 (splitk_gemm_fits).
bool splitk_gemm_fits(int M, int N, int K);
int splitk_ksplit(int N, int K);
void splitk_gemm(const f16* Afrag, const f16* Afrag_lo, const f16* Wp, float* part, int M, int N, int K, int ksplit,
                 int plane_rows, int prow0, hipStream_t st);
void reduce_resid_norm(const float* part, int ksplit, int plane_rows, int prow0, int M, int d, float* x,
                       const float* gain, float eps, f16* hn_frag, f16* hn_frag_lo, int row0, hipStream_t st);
void rmsnorm_frag(const float* x, int M, int d, const float* gain, float eps, f16* hn_frag, f16* hn_frag_lo,
                  hipStream_t st);
void reduce_swiglu(const float* part, int ksplit, int plane_rows, int prow0, int M, int f, f16* act_frag,
                   f16* act_frag_lo, int row0, hipStream_t st);

// Decode attention of the 16-bit path (one query per row of the step); output in fragment order.  k_lo / v_lo
// != nullptr: two-term mode (low terms of the cache, output also as low-term fragments out_frag_lo).
void decode_attention_fused(const float* part, int ksplit, int part_rows, const float* rope_cos, const float* rope_sin,
                            f16* k_cache, f16* v_cache, unsigned char* k_lo, unsigned char* v_lo, const int32_t* tok_seq,
                            const int32_t* tok_pos, f16* out_frag, f16* out_frag_lo, int B, int d_model, int n_heads,
                            int head_dim, int max_seq, hipStream_t st);

// Action head: final RMSNorm + action rows of the LM head -> logits [B, A] float32.
template <class T>
void head_logits(const float* x, const int32_t* row_index, const float* gain, const T* w_head,
                 float* logits, int ld_logits, int B, int d, int A, float eps, hipStream_t st);
void select_tokens(const float* logits, int ld_logits, int B, int A, float temperature, const float* gumbel, int k,
                   int n_tokens, const float* act_scale, const float* act_offset, int action_dim,
                   int32_t* tokens_out, float* logp_out, float* actions_out, int out_stride,
                   int32_t* next_ids, int id0, hipStream_t st);

// Value head (attention pooling over the rows that feed the action head, step embedding, GELU MLP).
void value_accumulate(const float* x, const int32_t* row_index, const float* gain, float eps, const float* attn_w,
                      const float* attn_b, int B, int d, bool first, float* vz, float* vml, hipStream_t st);
template <class T>
void value_finish(const float* vz, const float* vml, const T* step_emb, int n_steps, const int32_t* step_t,
                  const T* w1, const float* b1, const float* w2, const float* b2, int B, int d, float* vu, float* vh,
                  float* values, hipStream_t st);

// Last prefill layer, compact rows: gather attention output (to fragment order) and residual rows, scatter back.
// att_frag_lo != nullptr: att rows are [hi | lo] (pitch ld_att; lo8: the low terms are bytes), the low terms go to
// att_frag_lo as half precision
void gather_tail(const f16* att, int ld_att, bool lo8, const float* x, const int32_t* need, int n, int d,
                 f16* att_frag, f16* att_frag_lo, float* x_c, hipStream_t st);
void scatter_tail(const float* x_c, const int32_t* need, int n, int d, float* x, hipStream_t st);

// Chunk pass (all K action rows in one forward): merged id stream, fed-token buffer, emitting rows, scoring.
void merge_tail_ids(const int32_t* instr_ids, const int32_t* cu2_dev, const int32_t* tail, int B, int n_tail,
                    int total, int32_t* out, hipStream_t st);
void tail_ids(const int32_t* tokens, int B, int K, int id0, int A, int placeholder, int32_t* tail, hipStream_t st);
void chunk_rows(const int32_t* last_row, int B, int K, int32_t* rows, hipStream_t st);
void score_rows(const float* logits, int rows, int A, float temperature, const int32_t* tokens, const float* mu,
                float sigma, float* logp_out, float* ratio_out, float* weight_out, hipStream_t st);

// Ceiling probes (see vla_probe): an MFMA-only loop on weight bits and a plain streaming read.
void probe_mfma(const f16* w, size_t n_frag, int n_wg, int iters, float* sink, hipStream_t st);
void probe_stream(const void* src, size_t bytes, int n_wg, unsigned* sink, hipStream_t st);

// Small utilities.
void rope_table(float* cos_t, float* sin_t, int max_seq, int head_dim, float theta, hipStream_t st);
// slot_map: device [B] cache slot of each sequence of the call, nullptr = identity; seq_len is indexed by slot.
void build_token_maps(const int32_t* cu_patch_dev, const int32_t* cu_instr_dev, const int32_t* slot_map, int B,
                      int T_tokens, int32_t* tok_seq, int32_t* tok_pos, int32_t* tok_src, int32_t* last_row,
                      int32_t* seq_len, hipStream_t st);
void decode_maps(int32_t* seq_len, const int32_t* slot_map, int B, int32_t* tok_seq, int32_t* tok_pos, hipStream_t st);
void advance_lengths(int32_t* seq_len, const int32_t* slot_map, int B, hipStream_t st);
template <class T>
void convert_copy(const T* src, float* dst, size_t n, hipStream_t st);   // gains -> float32
template <class T>
void plain_copy(const T* src, T* dst, size_t n, hipStream_t st);

}  // namespace vla
