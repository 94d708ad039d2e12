// C ABI of the VLA policy library: context, validation, weight repacking and the host-side
// orchestration of prefill, decode step and policy step.  All device work is enqueued on the
// caller's stream; nothing here synchronises the device except the profiling read-out and vla_probe.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/vla.h"
#include "../../include/vla_bench.h"
#include "common.h"

using namespace vla;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// Staging memory of vla_decode_step_static: one array per GPU, part of the loaded code object, so that entry
// point needs no caller-provided or allocated staging.  Host code never uses the array's name as an address:
// static_scratch() asks the runtime once per device for the device address and keeps it.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
constexpr int kMaxDevices = 64;

struct LayerW {
  size_t g_attn, w_qkv, w_o, g_ffn, w_gu, w_down;   // byte offsets into the weight arena
  size_t w_qkv8, w_o8, w_gu8, w_down8;              // 8-bit copies for 8-bit low terms (two-term layers), else unused
};
struct ArenaLayout {
  size_t embed, g_final, head, total;
  size_t v_attn_w, v_attn_b, v_step_emb, v_w1, v_b1, v_w2, v_b2;   // value head (only if value_max_steps > 0)
  std::vector<LayerW> layers;
};
struct WorkLayout {
  size_t x, hn, q, att, act, scratch, part, rope_cos, rope_sin, tok_seq, tok_pos, tok_src, last_row, seq_len,
      cu_patch, cu_instr, cur_ids, logits, vz, vml, vu, vh, ids2, tail, chunk_rows, chunk_logits, slot_map, range_flag,
      total;
};

size_t elem_size(int dtype) { return dtype == VLA_BF16 ? 2 : 4; }

// High-precision mode of the 16-bit path: in the leading layers the activations that feed a matrix core, and the
// cached keys and values, are carried as hi + lo terms (two-term layers); buffers are sized for two terms.
inline bool two_term(const vla_config& c) { return c.dtype == VLA_BF16 && c.precision == VLA_PREC_HIGH; }
// ... in the leading layers only: nearly all of the logit error that single-term operands cause enters in the
// first few layers (the rounding model: rounding every operand from layer 4 on leaves 18 % of the rms error of
// rounding everywhere, from layer 2 on 25 %), so the layers after them run single-term.
constexpr int kDefaultTwoTermLayers = 4;
inline int two_term_layers(const vla_config& c) {
  if (!two_term(c)) return 0;
  const int n = c.two_term_layers > 0 ? c.two_term_layers : kDefaultTwoTermLayers;
  return n < c.n_layers ? n : c.n_layers;
}
inline bool two_term_layer(const vla_config& c, int l) { return l < two_term_layers(c); }
// Row-major two-term operands of the prefill GEMMs with contraction length K carry their low terms as bytes (and
// the GEMM uses the 8-bit copy of its weights for them) when K allows whole pairs of 64-k slabs; otherwise as
// half precision.  Row pitch of such an operand in halves; mode as the producing kernels take it.  `two`: whether
// the layer at hand is a two-term layer.
inline bool lo8(bool two, int K) { return two && K % 128 == 0; }
inline int lo_mode(bool two, int K) { return !two ? 0 : (lo8(two, K) ? 2 : 1); }
inline int two_pitch(bool two, int K) { return !two ? K : (lo8(two, K) ? K + K / 2 : 2 * K); }

ArenaLayout arena_layout(const vla_config& c) {
  ArenaLayout a;
  const size_t es = elem_size(c.dtype), d = c.d_model, f = c.d_ffn;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  a.embed = take((size_t)c.vocab * d * es);
  a.layers.resize(c.n_layers);
  int li = 0;
  for (auto& l : a.layers) {
    const bool two = two_term_layer(c, li++);
    l.g_attn = take(d * 4);
    l.w_qkv = take(3 * d * d * es);
    l.w_o = take(d * d * es);
    l.g_ffn = take(d * 4);
    l.w_gu = take(2 * f * d * es);
    l.w_down = take(d * f * es);
    l.w_qkv8 = take(lo8(two, (int)d) ? 3 * d * d : 0);
    l.w_o8 = take(lo8(two, (int)d) ? d * d : 0);
    l.w_gu8 = take(lo8(two, (int)d) ? 2 * f * d : 0);
    l.w_down8 = take(lo8(two, (int)f) ? d * f : 0);
  }
  a.g_final = take(d * 4);
  a.head = take((size_t)c.n_action_bins * d * es);
  if (c.value_max_steps > 0) {
    a.v_attn_w = take(d * 4);
    a.v_attn_b = take(4);
    a.v_step_emb = take((size_t)c.value_max_steps * d * es);
    a.v_w1 = take(d * d * es);
    a.v_b1 = take(d * 4);
    a.v_w2 = take(d * 4);
    a.v_b2 = take(4);
  }
  a.total = off;
  return a;
}
// Positions per (slot, head) block of the KV cache.  Kept odd: the blocks of the (slot, head) pairs that are
// streamed concurrently then start an odd number of 256-byte rows apart and spread over all memory channels
// (with max_seq = 608 the prefill attention of a 128 x 552-token batch took 1222 us per layer, with 609 1078 us).
inline int kv_pitch(const vla_config& c) { return c.max_seq | 1; }


size_t kv_layer_stride(const vla_config& c) {   // elements of K (or V) of one layer
  return (size_t)c.max_batch * c.n_heads * kv_pitch(c) * c.head_dim;
}
// one set of planes [layer][K|V][slot][head][position][head_dim]; a second set, for the two-term layers only, holds
// the low terms
size_t kv_plane_bytes(const vla_config& c) { return 2 * (size_t)c.n_layers * kv_layer_stride(c) * elem_size(c.dtype); }
size_t kv_lo_bytes(const vla_config& c) { return 2 * (size_t)two_term_layers(c) * kv_layer_stride(c); }   // one byte each
size_t kv_bytes(const vla_config& c) { return kv_plane_bytes(c) + align_up(kv_lo_bytes(c)); }

size_t max_rows(const vla_config& c) {
  const size_t b32 = ((size_t)c.max_batch + 31) / 32 * 32;   // fragment-order activations come in 32-row blocks
  return (size_t)c.max_prefill_tokens > b32 ? (size_t)c.max_prefill_tokens : b32;
}
constexpr int kMaxChunk = 64;         // most action tokens per sequence in the one-pass (chunk) entry points
// rows of one partial plane of the weight-streaming GEMMs: the whole decode batch, or one chunk of the last
// prefill layer's compact rows
size_t part_rows(const vla_config& c) {
  const size_t b32 = ((size_t)c.max_batch + 31) / 32 * 32;
  return b32 > 128 ? b32 : 128;
}

WorkLayout work_layout(const vla_config& c) {
  WorkLayout w;
  const size_t es = elem_size(c.dtype), d = c.d_model, f = c.d_ffn, T = max_rows(c), B = c.max_batch;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  const size_t terms = two_term(c) ? 2 : 1;      // two-term layers: rows [hi | lo], or a second set of fragment blocks
  w.x = take(T * d * 4);
  w.hn = take(T * d * es * terms);
  w.q = take(T * d * es * terms);
  w.att = take(T * d * es * terms);
  w.act = take(T * f * es * terms);
  const size_t widest = 3 * d > 2 * f ? 3 * d : 2 * f;
  w.scratch = take(c.dtype == VLA_F32 ? T * widest * 4 : 0);
  w.part = take(c.dtype == VLA_BF16 ? (size_t)kMaxKSplit * part_rows(c) * widest * 4 : 0);
  w.rope_cos = take((size_t)c.max_seq * (c.head_dim / 2) * 4);
  w.rope_sin = take((size_t)c.max_seq * (c.head_dim / 2) * 4);
  w.tok_seq = take(T * 4);
  w.tok_pos = take(T * 4);
  w.tok_src = take(T * 4);
  w.last_row = take(B * 4);
  w.seq_len = take(B * 4);
  w.cu_patch = take((B + 1) * 4);
  w.cu_instr = take((B + 1) * 4);
  w.cur_ids = take(B * 4);
  w.logits = take(B * (size_t)c.n_action_bins * 4);
  const size_t vrows = c.value_max_steps > 0 ? B : 0;
  w.vz = take(vrows * d * 4);
  w.vml = take(vrows * 2 * 4);
  w.vu = take(vrows * d * 4);
  w.vh = take(vrows * d * 4);
  w.ids2 = take(T * 4);
  w.tail = take(B * (size_t)kMaxChunk * 4);
  w.chunk_rows = take(B * (size_t)kMaxChunk * 4);
  w.chunk_logits = take(B * (size_t)kMaxChunk * c.n_action_bins * 4);
  w.slot_map = take(B * 4);
  w.range_flag = take(4);
  w.total = off;
  return w;
}

const char* check_config(const vla_config& c) {
  if (c.n_layers <= 0 || c.d_model <= 0 || c.n_heads <= 0 || c.head_dim <= 0 || c.d_ffn <= 0) return "non-positive model dimension";
  if ((int64_t)c.n_heads * c.head_dim != c.d_model) return "n_heads * head_dim must equal d_model";
  if (c.vocab <= 0 || c.n_action_bins <= 0 || c.n_action_bins > c.vocab) return "need 0 < n_action_bins <= vocab";
  if (c.n_action_bins > 1024) return "n_action_bins > 1024";
  if (c.dtype != VLA_F32 && c.dtype != VLA_BF16) return "dtype must be VLA_F32 or VLA_BF16";
  if (!(c.rope_theta > 0.f) || !(c.rms_eps >= 0.f)) return "rope_theta must be > 0 and rms_eps >= 0";
  if (c.max_batch <= 0 || c.max_seq <= 0 || c.max_prefill_tokens <= 0) return "capacities must be positive";
  if (c.value_max_steps < 0) return "value_max_steps must be >= 0";
  if (c.precision != VLA_PREC_HIGH && c.precision != VLA_PREC_FAST) return "precision must be VLA_PREC_HIGH or VLA_PREC_FAST";
  if (c.two_term_layers < 0) return "two_term_layers must not be negative";
  if (c.head_dim != 32 && c.head_dim != 64 && c.head_dim != 128 && c.head_dim != 256) return "head_dim must be 32, 64, 128 or 256";
  if (c.d_model % 4) return "d_model must be a multiple of 4";
  if (c.dtype == VLA_BF16) {
    if (c.head_dim != 64 && c.head_dim != 128) return "bf16 path needs head_dim 64 or 128";
    if (c.d_model % 128 || c.d_ffn % 64) return "bf16 path needs d_model % 128 == 0 and d_ffn % 64 == 0";
  }
  if (c.dtype == VLA_F32 && (size_t)(c.head_dim + kv_pitch(c)) * 16 > 64 * 1024)
    return "max_seq too large for the float32 attention kernel's LDS";
  if ((int64_t)c.d_model * 4 > 64 * 1024) return "d_model too large for the head kernel's LDS";
  return nullptr;
}

struct EventPair { hipEvent_t a, b; };

}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of this GPU's copy of `scratch` (looked up on the first call per device, with that device current).
hipError_t static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}
}  // namespace

struct vla_ctx {
  vla_config cfg;
  ArenaLayout al;
  WorkLayout wl;
  char* arena = nullptr;
  char* kv = nullptr;
  char* work = nullptr;
  bool bound = false, weights = false, tables = false, value_weights = false;
  // serving state of the in-place weight update (accepting -> draining -> updating -> accepting)
  int serving = VLA_ACCEPTING;
  int64_t version = 0;               // bumped by every completed load / update
  hipEvent_t ev_work = nullptr;      // recorded after the last compute call, on its stream
  hipEvent_t ev_update = nullptr;    // recorded when the last load / update was committed, on its stream
  bool have_work = false, have_update = false;
  int active_B = 0;                  // batch of the last prefill (0: none)
  int run_B = 0, run_max_len = 0;    // batch and longest prefix of the prefill being enqueued
  const int32_t* run_slots = nullptr; // device slot map of the call being enqueued (nullptr: sequence b is slot b)
  float* part_override = nullptr;    // set for the duration of vla_decode_step_static: GEMM staging outside the workspace
  std::vector<int32_t> len;          // host copy of the sequence lengths
  std::string err;
  // pinned staging ring for the host offset arrays
  static constexpr int kRing = 8;
  int32_t* stage = nullptr;
  // weight range check of the 16-bit path: the pack kernels OR bits into a device flag, a copy to range_host
  // (pinned) follows every load / update, and the first compute call that finds the copy complete reports it
  int32_t* range_host = nullptr;
  bool range_pending = false, weights_bad = false;
  hipEvent_t stage_ev[kRing];
  bool stage_used[kRing];
  int stage_next = 0;
  // profiling
  unsigned prof_mask = 0;
  std::vector<EventPair> prof[FAM_COUNT];
  std::vector<hipEvent_t> ev_pool;
};

namespace {

int fail(vla_ctx* ctx, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (ctx) ctx->err = buf;
  return code;
}

#define HIP_TRY(ctx, expr)                                                                       \
  do {                                                                                           \
    hipError_t e_ = (expr);                                                                      \
    if (e_ != hipSuccess) return fail(ctx, VLA_E_HIP, "%s: %s", #expr, hipGetErrorString(e_));   \
  } while (0)

struct ProfScope {
  vla_ctx* c;
  int fam;
  hipStream_t st;
  EventPair p;
  bool on;
  ProfScope(vla_ctx* c_, int fam_, hipStream_t st_) : c(c_), fam(fam_), st(st_), on((c_->prof_mask >> fam_) & 1u) {
    if (!on) return;
    if (hipEventCreate(&p.a) != hipSuccess || hipEventCreate(&p.b) != hipSuccess) { on = false; return; }
    (void)hipEventRecord(p.a, st);
  }
  ~ProfScope() {
    if (!on) return;
    (void)hipEventRecord(p.b, st);
    c->prof[fam].push_back(p);
  }
};

const char* kFamilyNames[FAM_COUNT] = {"gemm_qkv_prefill", "gemm_o_prefill", "gemm_gateup_prefill",
                                       "gemm_down_prefill", "attn_prefill", "gemm_qkv_decode", "gemm_o_decode",
                                       "gemm_gateup_decode", "gemm_down_decode", "attn_decode", "rmsnorm",
                                       "head_select", "misc", "prefill_tail", "gemm_qkv_two_prefill",
                                       "gemm_o_two_prefill", "gemm_gateup_two_prefill", "gemm_down_two_prefill"};

template <class T> T* at(char* base, size_t off) { return reinterpret_cast<T*>(base + off); }

// ---- one pass over the layers for `rows` packed tokens (prefill: all prefix tokens; decode: B) ------
// T is the activation type: f16 on the 16-bit path (bf16 storage), float on the float32 path.
void run_tail_f16(vla_ctx* ctx, const LayerW& lw, const int32_t* need, int n_need, hipStream_t st);

RopeKv layer_rope_kv(vla_ctx* ctx, int l) {
  const vla_config& c = ctx->cfg;
  const WorkLayout& w = ctx->wl;
  const size_t es = elem_size(c.dtype), kvl = kv_layer_stride(c) * es;   // bytes of K (or V) of one layer
  const bool two = two_term_layer(c, l);
  RopeKv rk;
  rk.q = ctx->work + w.q;
  rk.k_cache = ctx->kv + (size_t)(2 * l) * kvl;
  rk.v_cache = ctx->kv + (size_t)(2 * l + 1) * kvl;
  rk.k_lo = two ? ctx->kv + kv_plane_bytes(c) + (size_t)(2 * l) * kv_layer_stride(c) : nullptr;
  rk.v_lo = two ? ctx->kv + kv_plane_bytes(c) + (size_t)(2 * l + 1) * kv_layer_stride(c) : nullptr;
  rk.ldq = two ? 2 * c.d_model : c.d_model;
  rk.tok_seq = at<int32_t>(ctx->work, w.tok_seq);
  rk.tok_pos = at<int32_t>(ctx->work, w.tok_pos);
  rk.rope_cos = at<float>(ctx->work, w.rope_cos);
  rk.rope_sin = at<float>(ctx->work, w.rope_sin);
  rk.n_heads = c.n_heads;
  rk.head_dim = c.head_dim;
  rk.max_seq = kv_pitch(c);
  rk.d_model = c.d_model;
  return rk;
}

// need / n_need (prefill only): the packed rows whose final hidden state is read afterwards.  When they are
// few, the last layer's output projection and feed-forward run on those rows alone.
// Two-term layers (16-bit path, the leading layers of the high-precision mode): the normalised rows that feed the
// QKV and the gate/up GEMMs, q / k / v, the attention output and the SwiGLU output are carried as [hi | lo].
template <class T>
int run_layers(vla_ctx* ctx, int rows, bool decode, hipStream_t st, const int32_t* need = nullptr, int n_need = 0) {
  const vla_config& c = ctx->cfg;
  const WorkLayout& w = ctx->wl;
  const int d = c.d_model, f = c.d_ffn;
  const f16* no8 = nullptr;
  float* x = at<float>(ctx->work, w.x);
  T* hn = at<T>(ctx->work, w.hn);
  T* q = at<T>(ctx->work, w.q);
  T* att = at<T>(ctx->work, w.att);
  T* act = at<T>(ctx->work, w.act);
  float* gemm_out = ctx->part_override ? ctx->part_override : at<float>(ctx->work, w.scratch);
  const int32_t* tok_seq = at<int32_t>(ctx->work, w.tok_seq);
  const int32_t* tok_pos = at<int32_t>(ctx->work, w.tok_pos);
  const int fam_attn = decode ? FAM_ATTN_DECODE : FAM_ATTN_PREFILL;
  for (int l = 0; l < c.n_layers; ++l) {
    const LayerW& lw = ctx->al.layers[l];
    const RopeKv rk = layer_rope_kv(ctx, l);
    const bool two = two_term_layer(c, l);
    const int pd = two_pitch(two, d), pf = two_pitch(two, f);     // row pitch of this layer's operands with K = d, f
    const int fam_gemm = decode ? FAM_GEMM_QKV_DECODE                  // + 0 qkv, 1 o, 2 gate-up, 3 down
                                : (two ? FAM_GEMM_QKV_TWO_PREFILL : FAM_GEMM_QKV_PREFILL);
    {
      ProfScope ps(ctx, FAM_NORM, st);
      rmsnorm<T>(x, nullptr, at<float>(ctx->arena, lw.g_attn), hn, rows, d, c.rms_eps, nullptr, lo_mode(two, d), st);
    }
    {
      ProfScope ps(ctx, fam_gemm + 0, st);
      if constexpr (sizeof(T) == 2) {
        gemm_f16_qkv(GemmF16{(const f16*)hn, pd, at<f16>(ctx->arena, lw.w_qkv), rows, 3 * d, pd, d,
                             lo8(two, d) ? at<f16>(ctx->arena, lw.w_qkv8) : no8}, rk, st);
      } else {
        gemm_f32((const float*)hn, d, at<float>(ctx->arena, lw.w_qkv), gemm_out, rows, 3 * d, d, st);
        rope_kv_f32(gemm_out, rows, rk, st);
      }
    }
    {
      ProfScope ps(ctx, fam_attn, st);
      if constexpr (sizeof(T) == 2) {
        flash_prefill((const f16*)q, rk.ldq, (const f16*)rk.k_cache, (const f16*)rk.v_cache, (const unsigned char*)rk.k_lo,
                      (const unsigned char*)rk.v_lo, at<int32_t>(ctx->work, w.cu_patch), at<int32_t>(ctx->work, w.cu_instr),
                      ctx->run_slots, (f16*)att, pd, lo8(two, d), ctx->run_B, ctx->run_max_len, c.n_heads, c.head_dim,
                      kv_pitch(c), st);
      } else {
        attention_rows<T>(q, d, (const T*)rk.k_cache, (const T*)rk.v_cache, tok_seq, tok_pos, att, d, rows,
                          c.n_heads, c.head_dim, kv_pitch(c), false, st);
      }
    }
    if constexpr (sizeof(T) == 2) {
      // the compact set lives in buffers that are dead by now (see run_tail_f16): it must fit them
      const size_t pad32 = ((size_t)n_need + 31) / 32 * 32;
      const bool fits = pad32 <= max_rows(c) &&
                        align_up(pad32 * f * sizeof(f16)) + (size_t)n_need * d * 4 <= max_rows(c) * (size_t)f * sizeof(f16);
      if (!decode && l == c.n_layers - 1 && need && n_need > 0 && (size_t)n_need * 2 <= (size_t)rows && fits) {
        run_tail_f16(ctx, lw, need, n_need, st);
        break;
      }
    }
    {
      ProfScope ps(ctx, fam_gemm + 1, st);
      if constexpr (sizeof(T) == 2) {
        gemm_f16_resid(GemmF16{(const f16*)att, pd, at<f16>(ctx->arena, lw.w_o), rows, d, pd, d,
                               lo8(two, d) ? at<f16>(ctx->arena, lw.w_o8) : no8}, x, d, st);
      } else {
        gemm_f32((const float*)att, d, at<float>(ctx->arena, lw.w_o), gemm_out, rows, d, d, st);
        resid_add_f32(x, gemm_out, (size_t)rows * d, st);
      }
    }
    {
      ProfScope ps(ctx, FAM_NORM, st);
      rmsnorm<T>(x, nullptr, at<float>(ctx->arena, lw.g_ffn), hn, rows, d, c.rms_eps, nullptr, lo_mode(two, d), st);
    }
    {
      ProfScope ps(ctx, fam_gemm + 2, st);
      if constexpr (sizeof(T) == 2) {
        gemm_f16_swiglu(GemmF16{(const f16*)hn, pd, at<f16>(ctx->arena, lw.w_gu), rows, 2 * f, pd, d,
                                lo8(two, d) ? at<f16>(ctx->arena, lw.w_gu8) : no8}, (f16*)act, pf, lo_mode(two, f), st);
      } else {
        gemm_f32((const float*)hn, d, at<float>(ctx->arena, lw.w_gu), gemm_out, rows, 2 * f, d, st);
        swiglu_f32(gemm_out, (float*)act, rows, f, st);
      }
    }
    {
      ProfScope ps(ctx, fam_gemm + 3, st);
      if constexpr (sizeof(T) == 2) {
        gemm_f16_resid(GemmF16{(const f16*)act, pf, at<f16>(ctx->arena, lw.w_down), rows, d, pf, f,
                               lo8(two, f) ? at<f16>(ctx->arena, lw.w_down8) : no8}, x, d, st);
      } else {
        gemm_f32((const float*)act, f, at<float>(ctx->arena, lw.w_down), gemm_out, rows, d, f, st);
        resid_add_f32(x, gemm_out, (size_t)rows * d, st);
      }
    }
  }
  return VLA_OK;
}

// Fragment-order activations of the weight-streaming GEMMs: block row r0/32 of an [M, K] operand, and in two-term
// mode the matching low-term blocks, kept max_rows * K elements further on in the same buffer.
inline f16* frag_rows(f16* base, int row0, int K) { return base + (size_t)(row0 / 32) * (K / 16) * 512; }
// (nullptr when no layer is a two-term layer; single-term layers of a two-term configuration pass nullptr on)
inline f16* frag_lo(const vla_config& c, f16* base, int K) { return two_term(c) ? base + max_rows(c) * (size_t)K : nullptr; }

// Decode step of the 16-bit path: split-K GEMMs whose partial planes span the whole batch, and one kernel after each
// GEMM that sums the planes and applies the elementwise step for all rows.  Batches of up to kSkinnyMaxRows rows
// use the weight-streaming kernel (every wave an independent stream; a 128-row accumulator tile is what a wave's
// registers hold without spilling).  Larger batches send their wide matrices through the 256 x 256 tiled kernel in
// chunks of 256 rows, split over K (activations shared through LDS, every weight read once per 256 rows); a
// remainder of at most 128 rows, and the matrices the tiled kernel does not take, go to the weight-streaming
// kernel in chunks of 128 rows with the same number of planes (the later chunks find the matrix they re-read in
// the 256 MB last-level cache).
int run_layers_decode_f16(vla_ctx* ctx, int B, hipStream_t st) {
  const vla_config& c = ctx->cfg;
  const WorkLayout& w = ctx->wl;
  const int d = c.d_model, f = c.d_ffn;
  float* x = at<float>(ctx->work, w.x);
  f16* hn = at<f16>(ctx->work, w.hn);
  f16* att = at<f16>(ctx->work, w.att);
  f16* act = at<f16>(ctx->work, w.act);
  f16 *hn_lo = frag_lo(c, hn, d), *att_lo = frag_lo(c, att, d), *act_lo = frag_lo(c, act, f);
  float* part = ctx->part_override ? ctx->part_override : at<float>(ctx->work, w.part);
  // the tiled split-K kernel takes the chunks of more than 128 rows of the wide matrices (QKV, gate/up at 7B): it
  // needs about half the compute units busy to beat two weight-streaming launches (measured at 256 rows on the 7B
  // shape: QKV 44 against 74 us, gate/up 82 against 122; but the N = 4096 projections, 64 workgroups, 46 and 83
  // against 45 and 72)
  // (matrices of up to 2 M elements are launch-bound either way: one tiled launch per 256 rows instead of two)
  auto tiled = [&](int N, int K) {
    return B > kSkinnyMaxRows && splitk_gemm_fits(256, N, K) &&
           ((N / 256) * splitk_ksplit(N, K) >= 128 || (size_t)N * K <= ((size_t)2 << 20));
  };
  auto planes = [&](int N, int K) { return tiled(N, K) ? splitk_ksplit(N, K) : skinny_ksplit(N, K); };
  const int ks_qkv = planes(3 * d, d), ks_o = planes(d, d), ks_gu = planes(2 * f, d), ks_dn = planes(d, f);
  auto gemm = [&](f16* a, f16* a_lo, size_t w_off, int N, int K, int ks) {
    int r0 = 0;
    if (tiled(N, K)) {
      for (; B - r0 > kSkinnyMaxRows; r0 += 256) {
        const int m = B - r0 < 256 ? B - r0 : 256;
        splitk_gemm(frag_rows(a, r0, K), a_lo ? frag_rows(a_lo, r0, K) : nullptr, at<f16>(ctx->arena, w_off), part, m,
                    N, K, ks, B, r0, st);
      }
    }
    for (; r0 < B; r0 += kSkinnyMaxRows) {
      const int m = B - r0 < kSkinnyMaxRows ? B - r0 : kSkinnyMaxRows;
      skinny_gemm(frag_rows(a, r0, K), a_lo ? frag_rows(a_lo, r0, K) : nullptr, at<f16>(ctx->arena, w_off), part, m, N, K,
                  ks, B, r0, st);
    }
  };
  f16* const none = nullptr;
  {
    ProfScope ps(ctx, FAM_NORM, st);
    rmsnorm_frag(x, B, d, at<float>(ctx->arena, ctx->al.layers[0].g_attn), c.rms_eps, hn,
                 two_term_layer(c, 0) ? hn_lo : none, st);
  }
  for (int l = 0; l < c.n_layers; ++l) {
    const LayerW& lw = ctx->al.layers[l];
    const RopeKv rk = layer_rope_kv(ctx, l);      // low-term planes only in two-term layers
    const bool two = two_term_layer(c, l), two_next = two_term_layer(c, l + 1);
    {
      ProfScope ps(ctx, FAM_GEMM_QKV_DECODE, st);
      gemm(hn, two ? hn_lo : none, lw.w_qkv, 3 * d, d, ks_qkv);
    }
    {
      // the attention kernel itself sums the QKV partials of its (sequence, head), applies RoPE and appends the
      // new cache row
      ProfScope ps(ctx, FAM_ATTN_DECODE, st);
      decode_attention_fused(part, ks_qkv, B, rk.rope_cos, rk.rope_sin, (f16*)rk.k_cache, (f16*)rk.v_cache,
                             (unsigned char*)rk.k_lo, (unsigned char*)rk.v_lo, rk.tok_seq, rk.tok_pos, att, two ? att_lo : none, B, d,
                             c.n_heads, c.head_dim,
                             kv_pitch(c), st);
    }
    {
      ProfScope ps(ctx, FAM_GEMM_O_DECODE, st);
      gemm(att, two ? att_lo : none, lw.w_o, d, d, ks_o);
      reduce_resid_norm(part, ks_o, B, 0, B, d, x, at<float>(ctx->arena, lw.g_ffn), c.rms_eps, hn, two ? hn_lo : none, 0,
                        st);
    }
    {
      ProfScope ps(ctx, FAM_GEMM_GATEUP_DECODE, st);
      gemm(hn, two ? hn_lo : none, lw.w_gu, 2 * f, d, ks_gu);
      reduce_swiglu(part, ks_gu, B, 0, B, f, act, two ? act_lo : none, 0, st);
    }
    {
      ProfScope ps(ctx, FAM_GEMM_DOWN_DECODE, st);
      const float* next_gain = l + 1 < c.n_layers ? at<float>(ctx->arena, ctx->al.layers[l + 1].g_attn) : nullptr;
      gemm(act, two ? act_lo : none, lw.w_down, d, f, ks_dn);
      reduce_resid_norm(part, ks_dn, B, 0, B, d, x, next_gain, c.rms_eps, hn, two_next ? hn_lo : none, 0, st);
    }
  }
  return VLA_OK;
}

// Output projection and feed-forward of one layer for n_need compact rows with the weight-streaming GEMMs.
// Buffers that are dead at this point of the last prefill layer hold the compact set: q -> attention output in
// fragment order, hn -> normalised rows, act -> SwiGLU output followed by the float32 residual rows.
void run_tail_f16(vla_ctx* ctx, const LayerW& lw, const int32_t* need, int n_need, hipStream_t st) {
  const vla_config& c = ctx->cfg;
  const WorkLayout& w = ctx->wl;
  const int d = c.d_model, f = c.d_ffn;
  const bool two = two_term_layer(c, c.n_layers - 1);    // the layer this is the tail of
  ProfScope ps(ctx, FAM_TAIL, st);
  float* x = at<float>(ctx->work, w.x);
  f16* att = at<f16>(ctx->work, w.att);
  f16* att_frag = at<f16>(ctx->work, w.q);
  f16* hn = at<f16>(ctx->work, w.hn);
  f16* act = at<f16>(ctx->work, w.act);
  f16* const none = nullptr;
  f16* att_frag_lo = two ? frag_lo(c, att_frag, d) : none;
  f16* hn_lo = two ? frag_lo(c, hn, d) : none;
  f16* act_lo = two ? frag_lo(c, act, f) : none;
  float* part = at<float>(ctx->work, w.part);
  const size_t pad32 = ((size_t)n_need + 31) / 32 * 32;
  // the float32 residual rows of the compact set sit behind the SwiGLU fragments (hi, and lo in a two-term
  // layer: the lo blocks start max_rows * f elements in, so the rows go behind the whole buffer's used part)
  float* x_c = reinterpret_cast<float*>(reinterpret_cast<char*>(act) +
                                        (two ? max_rows(c) * (size_t)f * sizeof(f16) : 0) +
                                        align_up(pad32 * f * sizeof(f16)));
  const int ks_o = skinny_ksplit(d, d), ks_gu = skinny_ksplit(2 * f, d), ks_dn = skinny_ksplit(d, f);
  const int chunk = (int)(part_rows(c) < (size_t)kSkinnyMaxRows ? part_rows(c) : (size_t)kSkinnyMaxRows);
  gather_tail(att, two_pitch(two, d), lo8(two, d), x, need, n_need, d, att_frag, att_frag_lo, x_c, st);
  for (int r0 = 0; r0 < n_need; r0 += chunk) {
    const int m = n_need - r0 < chunk ? n_need - r0 : chunk;
    skinny_gemm(frag_rows(att_frag, r0, d), two ? frag_rows(att_frag_lo, r0, d) : nullptr, at<f16>(ctx->arena, lw.w_o),
                part, m, d, d, ks_o, m, 0, st);
    reduce_resid_norm(part, ks_o, m, 0, m, d, x_c, at<float>(ctx->arena, lw.g_ffn), c.rms_eps, hn, hn_lo, r0, st);
    skinny_gemm(frag_rows(hn, r0, d), two ? frag_rows(hn_lo, r0, d) : nullptr, at<f16>(ctx->arena, lw.w_gu), part, m,
                2 * f, d, ks_gu, m, 0, st);
    reduce_swiglu(part, ks_gu, m, 0, m, f, act, act_lo, r0, st);
    skinny_gemm(frag_rows(act, r0, f), two ? frag_rows(act_lo, r0, f) : nullptr, at<f16>(ctx->arena, lw.w_down), part, m, d,
                f, ks_dn, m, 0, st);
    reduce_resid_norm(part, ks_dn, m, 0, m, d, x_c, nullptr, c.rms_eps, hn, nullptr, r0, st);
  }
  scatter_tail(x_c, need, n_need, d, x, st);
}

template <class T>
void run_head(vla_ctx* ctx, int B, const int32_t* row_index, float* logits, int ld, hipStream_t st) {
  const vla_config& c = ctx->cfg;
  ProfScope ps(ctx, FAM_HEAD, st);
  head_logits<T>(at<float>(ctx->work, ctx->wl.x), row_index, at<float>(ctx->arena, ctx->al.g_final),
                 at<T>(ctx->arena, ctx->al.head), logits, ld, B, c.d_model, c.n_action_bins, c.rms_eps, st);
}

// One more row per sequence for the value head's attention pooling: the rows the action head just used.
void run_value_accumulate(vla_ctx* ctx, int B, const int32_t* row_index, bool first, hipStream_t st) {
  ProfScope ps(ctx, FAM_HEAD, st);
  value_accumulate(at<float>(ctx->work, ctx->wl.x), row_index, at<float>(ctx->arena, ctx->al.g_final), ctx->cfg.rms_eps,
                   at<float>(ctx->arena, ctx->al.v_attn_w), at<float>(ctx->arena, ctx->al.v_attn_b), B, ctx->cfg.d_model,
                   first, at<float>(ctx->work, ctx->wl.vz), at<float>(ctx->work, ctx->wl.vml), st);
}

// Result of the weight range check of the last load / update, once its device work has completed (wait: block
// until then).  Out-of-range weights make every compute call fail until a good set is loaded.
int poll_weight_range(vla_ctx* ctx, bool wait) {
  if (ctx->range_pending) {
    hipError_t e = wait ? hipEventSynchronize(ctx->ev_update) : hipEventQuery(ctx->ev_update);
    if (e == hipSuccess) {
      ctx->range_pending = false;
      ctx->weights_bad = *ctx->range_host != 0;
    } else if (e != hipErrorNotReady) {
      return fail(ctx, VLA_E_HIP, "weight range check: %s", hipGetErrorString(e));
    }
  }
  if (ctx->weights_bad)
    return fail(ctx, VLA_E_WEIGHTS, "a loaded weight matrix holds a value that the half-precision re-encoding cannot "
                "represent (|w| > 255 or not finite)");
  return VLA_OK;
}

int check_ready(vla_ctx* ctx) {
  if (!ctx->bound) return fail(ctx, VLA_E_STATE, "buffers are not bound (vla_bind_buffers)");
  if (!ctx->weights) return fail(ctx, VLA_E_STATE, "weights are not loaded (vla_load_weights)");
  return poll_weight_range(ctx, false);
}

// Start / end of the device work of a load or an update with respect to the range flag.
int range_check_begin(vla_ctx* ctx, hipStream_t st) {
  if (ctx->cfg.dtype != VLA_BF16) return VLA_OK;
  HIP_TRY(ctx, hipMemsetAsync(at<int32_t>(ctx->work, ctx->wl.range_flag), 0, 4, st));
  return VLA_OK;
}
int range_check_end(vla_ctx* ctx, hipStream_t st) {    // before the event that marks the end of the load is recorded
  if (ctx->cfg.dtype != VLA_BF16) return VLA_OK;
  HIP_TRY(ctx, hipMemcpyAsync(ctx->range_host, at<int32_t>(ctx->work, ctx->wl.range_flag), 4, hipMemcpyDeviceToHost, st));
  ctx->range_pending = true;
  return VLA_OK;
}

// Gate of every compute call.  A new batch is refused from the moment a drain was requested; steps of
// the batch in flight still run while draining; nothing runs while tensors are being overwritten.  The
// stream is made to wait (on the device) for the last committed update, whatever stream that ran on.
int check_serving(vla_ctx* ctx, bool new_batch) {
  if (ctx->serving == VLA_UPDATING) return fail(ctx, VLA_E_DRAINING, "weights are being updated (vla_update_commit ends it)");
  if (ctx->serving == VLA_DRAINING && new_batch)
    return fail(ctx, VLA_E_DRAINING, "draining for a weight update: no new batch is accepted");
  return VLA_OK;
}

int enter_compute(vla_ctx* ctx, hipStream_t st) {
  if (ctx->have_update) HIP_TRY(ctx, hipStreamWaitEvent(st, ctx->ev_update, 0));
  return VLA_OK;
}

int leave_compute(vla_ctx* ctx, hipStream_t st) {
  HIP_TRY(ctx, hipEventRecord(ctx->ev_work, st));
  ctx->have_work = true;
  return VLA_OK;
}

// Validates a prefill request and returns the packed token count.
int check_prefill(vla_ctx* ctx, int32_t B, const void* patch_emb, const int32_t* cu_patch,
                  const int32_t* instr_ids, const int32_t* cu_instr, int extra_positions, int64_t* T_out) {
  const vla_config& c = ctx->cfg;
  if (!cu_patch || !cu_instr) return fail(ctx, VLA_E_NULL, "cu_patch / cu_instr is NULL");
  if (B <= 0) return fail(ctx, VLA_E_SHAPE, "batch %d must be positive", B);
  if (B > c.max_batch) return fail(ctx, VLA_E_CAPACITY, "batch %d exceeds max_batch %d", B, c.max_batch);
  if (cu_patch[0] != 0 || cu_instr[0] != 0) return fail(ctx, VLA_E_SHAPE, "cumulative offsets must start at 0");
  int64_t T = 0;
  for (int b = 0; b < B; ++b) {
    const int np = cu_patch[b + 1] - cu_patch[b], li = cu_instr[b + 1] - cu_instr[b];
    if (np < 0 || li < 0) return fail(ctx, VLA_E_SHAPE, "offsets of sequence %d decrease", b);
    const int S = np + li;
    if (S < 1) return fail(ctx, VLA_E_SHAPE, "sequence %d has an empty prefix", b);
    if (S + extra_positions > c.max_seq)
      return fail(ctx, VLA_E_CAPACITY, "sequence %d needs %d positions, max_seq is %d", b, S + extra_positions, c.max_seq);
    T += S;
  }
  if (T > c.max_prefill_tokens)
    return fail(ctx, VLA_E_CAPACITY, "%lld prefix tokens exceed max_prefill_tokens %lld", (long long)T, (long long)c.max_prefill_tokens);
  if (cu_patch[B] > 0 && !patch_emb) return fail(ctx, VLA_E_NULL, "patch_emb is NULL");
  if (cu_instr[B] > 0 && !instr_ids) return fail(ctx, VLA_E_NULL, "instr_ids is NULL");
  *T_out = T;
  return VLA_OK;
}

int ensure_tables(vla_ctx* ctx, hipStream_t st) {
  if (ctx->tables) return VLA_OK;
  rope_table(at<float>(ctx->work, ctx->wl.rope_cos), at<float>(ctx->work, ctx->wl.rope_sin), ctx->cfg.max_seq,
             ctx->cfg.head_dim, ctx->cfg.rope_theta, st);
  ctx->tables = true;
  return VLA_OK;
}

template <class S> struct ActOf { typedef float type; };
template <> struct ActOf<bf16> { typedef f16 type; };

// S is the storage type of the caller's tensors (bf16 or float).
template <class T>
int do_prefill(vla_ctx* ctx, int32_t B, const void* patch_emb, const int32_t* cu_patch, const int32_t* instr_ids,
               const int32_t* cu_instr, int64_t T_tokens, float* logits, int ld_logits, hipStream_t st,
               const int32_t* tail = nullptr, int n_tail = 0, const int32_t* slots = nullptr) {
  const int n_last = n_tail + 1;   // rows per sequence whose final hidden state is read: the last n_tail + 1
  // slots (host, [B], or nullptr): cache slot of each sequence; nullptr means sequence b goes to slot b.
  // With a tail, cu_instr already counts n_tail extra ids per sequence (device array tail[B, n_tail]) and the
  // id stream the layers see is the merge of instr_ids and tail.
  const vla_config& c = ctx->cfg;
  const WorkLayout& w = ctx->wl;
  // stage the host offset arrays in pinned memory (a slot is reused only after its copy finished)
  const int slot = ctx->stage_next;
  ctx->stage_next = (slot + 1) % vla_ctx::kRing;
  if (ctx->stage_used[slot]) HIP_TRY(ctx, hipEventSynchronize(ctx->stage_ev[slot]));
  int32_t* host = ctx->stage + (size_t)slot * 3 * (c.max_batch + 1);
  memcpy(host, cu_patch, (B + 1) * sizeof(int32_t));
  memcpy(host + c.max_batch + 1, cu_instr, (B + 1) * sizeof(int32_t));
  HIP_TRY(ctx, hipMemcpyAsync(at<int32_t>(ctx->work, w.cu_patch), host, (B + 1) * 4, hipMemcpyHostToDevice, st));
  HIP_TRY(ctx, hipMemcpyAsync(at<int32_t>(ctx->work, w.cu_instr), host + c.max_batch + 1, (B + 1) * 4, hipMemcpyHostToDevice, st));
  ctx->run_slots = nullptr;
  if (slots) {
    memcpy(host + 2 * (c.max_batch + 1), slots, B * sizeof(int32_t));
    HIP_TRY(ctx, hipMemcpyAsync(at<int32_t>(ctx->work, w.slot_map), host + 2 * (c.max_batch + 1), B * 4, hipMemcpyHostToDevice, st));
    ctx->run_slots = at<int32_t>(ctx->work, w.slot_map);
  }
  HIP_TRY(ctx, hipEventRecord(ctx->stage_ev[slot], st));
  ctx->stage_used[slot] = true;
  ensure_tables(ctx, st);
  {
    ProfScope ps(ctx, FAM_MISC, st);
    build_token_maps(at<int32_t>(ctx->work, w.cu_patch), at<int32_t>(ctx->work, w.cu_instr), ctx->run_slots, B, (int)T_tokens,
                     at<int32_t>(ctx->work, w.tok_seq), at<int32_t>(ctx->work, w.tok_pos),
                     at<int32_t>(ctx->work, w.tok_src), at<int32_t>(ctx->work, w.last_row),
                     at<int32_t>(ctx->work, w.seq_len), st);
    if (n_tail > 0) {
      merge_tail_ids(instr_ids, at<int32_t>(ctx->work, w.cu_instr), tail, B, n_tail, cu_instr[B],
                     at<int32_t>(ctx->work, w.ids2), st);
      instr_ids = at<int32_t>(ctx->work, w.ids2);
    }
    assemble_prefix<T>((const T*)patch_emb, instr_ids, at<T>(ctx->arena, ctx->al.embed),
                       at<int32_t>(ctx->work, w.tok_src), at<float>(ctx->work, w.x), (int)T_tokens, c.d_model,
                       c.vocab, st);
  }
  ctx->run_B = B;
  ctx->run_max_len = 0;
  for (int b = 0; b < B; ++b) {
    const int S = (cu_patch[b + 1] - cu_patch[b]) + (cu_instr[b + 1] - cu_instr[b]);
    if (S > ctx->run_max_len) ctx->run_max_len = S;
  }
  const int32_t* need = at<int32_t>(ctx->work, w.last_row);
  if (n_last > 1) {
    ProfScope ps(ctx, FAM_MISC, st);
    chunk_rows(at<int32_t>(ctx->work, w.last_row), B, n_last, at<int32_t>(ctx->work, w.chunk_rows), st);
    need = at<int32_t>(ctx->work, w.chunk_rows);
  }
  run_layers<typename ActOf<T>::type>(ctx, (int)T_tokens, false, st, need, B * n_last);
  if (logits) run_head<T>(ctx, B, at<int32_t>(ctx->work, w.last_row), logits, ld_logits, st);
  HIP_TRY(ctx, hipGetLastError());
  // host mirror of the sequence lengths, by slot (0: free)
  if (!slots) {
    ctx->active_B = B;
    ctx->len.assign(c.max_batch, 0);
  } else {
    ctx->active_B = 0;             // slots are now managed one by one: vla_decode_slots, not vla_decode_step
    ctx->len.resize(c.max_batch, 0);
  }
  for (int b = 0; b < B; ++b)
    ctx->len[slots ? slots[b] : b] = (cu_patch[b + 1] - cu_patch[b]) + (cu_instr[b + 1] - cu_instr[b]);
  return VLA_OK;
}

template <class T>
int do_decode(vla_ctx* ctx, int32_t B, const int32_t* token_ids, float* logits, int ld_logits, hipStream_t st,
              const int32_t* slots = nullptr) {
  const vla_config& c = ctx->cfg;
  const WorkLayout& w = ctx->wl;
  const int32_t* slot_map = nullptr;
  if (slots) {      // host list of cache slots, one per row of this step
    const int slot = ctx->stage_next;
    ctx->stage_next = (slot + 1) % vla_ctx::kRing;
    if (ctx->stage_used[slot]) HIP_TRY(ctx, hipEventSynchronize(ctx->stage_ev[slot]));
    int32_t* host = ctx->stage + (size_t)slot * 3 * (c.max_batch + 1);
    memcpy(host, slots, B * sizeof(int32_t));
    HIP_TRY(ctx, hipMemcpyAsync(at<int32_t>(ctx->work, w.slot_map), host, B * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(ctx, hipEventRecord(ctx->stage_ev[slot], st));
    ctx->stage_used[slot] = true;
    slot_map = at<int32_t>(ctx->work, w.slot_map);
  }
  {
    ProfScope ps(ctx, FAM_MISC, st);
    embed_tokens<T>(token_ids, at<T>(ctx->arena, ctx->al.embed), at<float>(ctx->work, w.x), B, c.d_model, c.vocab, st);
    decode_maps(at<int32_t>(ctx->work, w.seq_len), slot_map, B, at<int32_t>(ctx->work, w.tok_seq), at<int32_t>(ctx->work, w.tok_pos), st);
  }
  if (sizeof(T) == 2) run_layers_decode_f16(ctx, B, st);
  else run_layers<typename ActOf<T>::type>(ctx, B, true, st);
  if (logits) run_head<T>(ctx, B, nullptr, logits, ld_logits, st);
  {
    ProfScope ps(ctx, FAM_MISC, st);
    advance_lengths(at<int32_t>(ctx->work, w.seq_len), slot_map, B, st);
  }
  HIP_TRY(ctx, hipGetLastError());
  for (int b = 0; b < B; ++b) ctx->len[slots ? slots[b] : b] += 1;
  return VLA_OK;
}

// One forward pass over [prefix ; K-1 fed tokens] per sequence, action logits [B, K, A] of the K emitting rows.
// stored == nullptr feeds `placeholder` everywhere, otherwise the vocabulary ids of stored[b, 0..K-2].
template <class T>
int do_chunk(vla_ctx* ctx, int32_t B, const void* patch_emb, const int32_t* cu_patch, const int32_t* instr_ids,
             const int32_t* cu_instr, int64_t T_prefix, int K, const int32_t* stored, int placeholder, float* logits,
             hipStream_t st) {
  const vla_config& c = ctx->cfg;
  const WorkLayout& w = ctx->wl;
  const int n_tail = K - 1, A = c.n_action_bins;
  std::vector<int32_t> cu2(B + 1);
  for (int b = 0; b <= B; ++b) cu2[b] = cu_instr[b] + b * n_tail;
  int32_t* tail = at<int32_t>(ctx->work, w.tail);
  {
    ProfScope ps(ctx, FAM_MISC, st);
    tail_ids(stored, B, K, c.vocab - A, A, placeholder, tail, st);
  }
  int rc = do_prefill<T>(ctx, B, patch_emb, cu_patch, instr_ids, cu2.data(), T_prefix + (int64_t)B * n_tail, nullptr, 0,
                         st, tail, n_tail);
  if (rc) return rc;
  // the emitting rows were listed by do_prefill (K > 1) or are the last rows (K == 1)
  const int32_t* rows = K > 1 ? at<int32_t>(ctx->work, w.chunk_rows) : at<int32_t>(ctx->work, w.last_row);
  run_head<T>(ctx, B * K, rows, logits, A, st);
  HIP_TRY(ctx, hipGetLastError());
  return VLA_OK;
}

// Shared validation of the one-pass entry points; returns the packed prefix token count.
int check_chunk(vla_ctx* ctx, int32_t B, const void* patch_emb, const int32_t* cu_patch, const int32_t* instr_ids,
                const int32_t* cu_instr, int32_t K, int64_t* T_out) {
  if (K <= 0 || K > kMaxChunk) return fail(ctx, VLA_E_SHAPE, "n_tokens must be in [1, %d]", kMaxChunk);
  int rc = check_prefill(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, K - 1, T_out);
  if (rc) return rc;
  if (*T_out + (int64_t)B * (K - 1) > ctx->cfg.max_prefill_tokens)
    return fail(ctx, VLA_E_CAPACITY, "%lld prefix + %lld fed tokens exceed max_prefill_tokens %lld", (long long)*T_out,
                (long long)B * (K - 1), (long long)ctx->cfg.max_prefill_tokens);
  return VLA_OK;
}

// Validates a host slot list: n entries, each in [0, max_batch), no duplicates.
int check_slots(vla_ctx* ctx, int32_t n, const int32_t* slots) {
  if (!slots) return fail(ctx, VLA_E_NULL, "slot_ids is NULL");
  if (n <= 0) return fail(ctx, VLA_E_SHAPE, "the number of slots must be positive");
  if (n > ctx->cfg.max_batch) return fail(ctx, VLA_E_CAPACITY, "%d slots exceed max_batch %d", n, ctx->cfg.max_batch);
  std::vector<char> seen(ctx->cfg.max_batch, 0);
  for (int i = 0; i < n; ++i) {
    if (slots[i] < 0 || slots[i] >= ctx->cfg.max_batch) return fail(ctx, VLA_E_SHAPE, "slot id %d outside [0, max_batch)", slots[i]);
    if (seen[slots[i]]) return fail(ctx, VLA_E_SHAPE, "slot id %d given twice", slots[i]);
    seen[slots[i]] = 1;
  }
  return VLA_OK;
}

int check_decode(vla_ctx* ctx, int32_t B, int steps) {
  if (ctx->active_B == 0) return fail(ctx, VLA_E_STATE, "decode before prefill");
  if (B != ctx->active_B) return fail(ctx, VLA_E_SHAPE, "decode batch %d differs from the prefilled batch %d", B, ctx->active_B);
  for (int b = 0; b < B; ++b)
    if (ctx->len[b] + steps > ctx->cfg.max_seq)
      return fail(ctx, VLA_E_CAPACITY, "sequence %d is full (%d of %d positions)", b, ctx->len[b], ctx->cfg.max_seq);
  return VLA_OK;
}

}  // namespace

// ---- exported functions --------------------------------------------------------------------------------
extern "C" {

int vla_create(const vla_config* cfg, vla_ctx** out) {
  if (!cfg || !out) return VLA_E_NULL;
  *out = nullptr;
  if (check_config(*cfg)) return VLA_E_CONFIG;
  vla_ctx* ctx = new vla_ctx();
  ctx->cfg = *cfg;
  ctx->al = arena_layout(*cfg);
  ctx->wl = work_layout(*cfg);
  for (int i = 0; i < vla_ctx::kRing; ++i) { ctx->stage_used[i] = false; ctx->stage_ev[i] = nullptr; }
  *out = ctx;
  return VLA_OK;
}

int vla_destroy(vla_ctx* ctx) {
  if (!ctx) return VLA_E_NULL;
  if (ctx->stage) (void)hipHostFree(ctx->stage);
  if (ctx->range_host) (void)hipHostFree(ctx->range_host);
  for (int i = 0; i < vla_ctx::kRing; ++i)
    if (ctx->stage_ev[i]) (void)hipEventDestroy(ctx->stage_ev[i]);
  if (ctx->ev_work) (void)hipEventDestroy(ctx->ev_work);
  if (ctx->ev_update) (void)hipEventDestroy(ctx->ev_update);
  for (auto& v : ctx->prof)
    for (auto& p : v) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
  delete ctx;
  return VLA_OK;
}

const char* vla_last_error(const vla_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int vla_query_sizes(const vla_config* cfg, size_t* weight_arena_bytes, size_t* kv_bytes_out, size_t* workspace_bytes) {
  if (!cfg) return VLA_E_NULL;
  if (check_config(*cfg)) return VLA_E_CONFIG;
  if (weight_arena_bytes) *weight_arena_bytes = arena_layout(*cfg).total;
  if (kv_bytes_out) *kv_bytes_out = kv_bytes(*cfg);
  if (workspace_bytes) *workspace_bytes = work_layout(*cfg).total;
  return VLA_OK;
}

int vla_bind_buffers(vla_ctx* ctx, void* weight_arena, void* kv, void* workspace) {
  if (!ctx) return VLA_E_NULL;
  if (!weight_arena || !kv || !workspace) return fail(ctx, VLA_E_NULL, "a buffer is NULL");
  if (((uintptr_t)weight_arena | (uintptr_t)kv | (uintptr_t)workspace) % kAlign)
    return fail(ctx, VLA_E_SHAPE, "buffers must be %zu-byte aligned", kAlign);
  if (!ctx->stage) {
    HIP_TRY(ctx, hipHostMalloc((void**)&ctx->stage, (size_t)vla_ctx::kRing * 3 * (ctx->cfg.max_batch + 1) * sizeof(int32_t), hipHostMallocDefault));
    HIP_TRY(ctx, hipHostMalloc((void**)&ctx->range_host, 64, hipHostMallocDefault));
    *ctx->range_host = 0;
    for (int i = 0; i < vla_ctx::kRing; ++i) HIP_TRY(ctx, hipEventCreateWithFlags(&ctx->stage_ev[i], hipEventDisableTiming));
    HIP_TRY(ctx, hipEventCreateWithFlags(&ctx->ev_work, hipEventDisableTiming));
    HIP_TRY(ctx, hipEventCreateWithFlags(&ctx->ev_update, hipEventDisableTiming));
  }
  ctx->arena = (char*)weight_arena;
  ctx->kv = (char*)kv;
  ctx->work = (char*)workspace;
  ctx->bound = true;
  ctx->weights = false;
  ctx->value_weights = false;
  ctx->tables = false;
  ctx->active_B = 0;
  ctx->len.assign(ctx->cfg.max_batch, 0);
  ctx->serving = VLA_ACCEPTING;
  ctx->have_work = ctx->have_update = false;
  ctx->range_pending = ctx->weights_bad = false;
  return VLA_OK;
}

}  // extern "C"

namespace {

const char* const kLeaves[9] = {"attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down"};
const char* const kValueNames[7] = {"value.attn_w", "value.attn_b", "value.step_emb", "value.w1",
                                    "value.b1",     "value.w2",     "value.b2"};

// Tensor slots: 0 embed, 1 final_norm, 2 lm_head, 3 + 9*l + leaf, then the seven value-head tensors.
int policy_slots(const vla_config& c) { return 3 + 9 * c.n_layers; }
int all_slots(const vla_config& c) { return policy_slots(c) + (c.value_max_steps > 0 ? 7 : 0); }

std::string slot_name(const vla_config& c, int s) {
  if (s == 0) return "embed";
  if (s == 1) return "final_norm";
  if (s == 2) return "lm_head";
  if (s < policy_slots(c)) return "layers." + std::to_string((s - 3) / 9) + "." + kLeaves[(s - 3) % 9];
  return kValueNames[s - policy_slots(c)];
}

// Maps every tensor to its slot and checks dtype and shape; nothing is enqueued.  slot[] must hold
// all_slots(cfg) null pointers on entry.
int parse_tensors(vla_ctx* ctx, const vla_tensor* tensors, int32_t n_tensors, std::vector<const vla_tensor*>& slot) {
  const vla_config& c = ctx->cfg;
  const int64_t d = c.d_model, f = c.d_ffn, V = c.vocab, A = c.n_action_bins;
  const int np = policy_slots(c);
  if (n_tensors < 0) return fail(ctx, VLA_E_SHAPE, "n_tensors is negative");
  for (int i = 0; i < n_tensors; ++i) {
    const vla_tensor& t = tensors[i];
    if (!t.name || !t.dev_ptr) return fail(ctx, VLA_E_NULL, "tensor %d has a NULL name or pointer", i);
    int s = -1;
    if (!strcmp(t.name, "embed")) s = 0;
    else if (!strcmp(t.name, "final_norm")) s = 1;
    else if (!strcmp(t.name, "lm_head")) s = 2;
    else if (!strncmp(t.name, "value.", 6)) {
      if (c.value_max_steps <= 0) return fail(ctx, VLA_E_CONFIG, "'%s': the context was created without a value head", t.name);
      for (int k = 0; k < 7; ++k)
        if (!strcmp(t.name, kValueNames[k])) s = np + k;
    } else {
      int l = -1, used = 0;
      if (sscanf(t.name, "layers.%d.%n", &l, &used) == 1 && used > 0 && l >= 0 && l < c.n_layers)
        for (int k = 0; k < 9; ++k)
          if (!strcmp(t.name + used, kLeaves[k])) s = 3 + 9 * l + k;
    }
    if (s < 0) return fail(ctx, VLA_E_WEIGHTS, "unknown tensor name '%s'", t.name);
    if (slot[s]) return fail(ctx, VLA_E_WEIGHTS, "tensor '%s' given twice", t.name);
    if (t.dtype != c.dtype) return fail(ctx, VLA_E_WEIGHTS, "tensor '%s' has dtype %d, config has %d", t.name, t.dtype, c.dtype);
    int64_t r = 0, k = 0;   // expected shape (k == 0: vector)
    if (s == 0) { r = V; k = d; }
    else if (s == 1) { r = d; }
    else if (s == 2) { r = (t.ndim == 2 && t.shape[0] == A) ? A : V; k = d; }
    else if (s < np) {
      switch ((s - 3) % 9) {
        case 0: case 5: r = d; break;
        case 1: case 2: case 3: case 4: r = d; k = d; break;
        case 6: case 7: r = f; k = d; break;
        default: r = d; k = f; break;
      }
    } else {
      const int64_t vr[7] = {d, 1, c.value_max_steps, d, d, d, 1}, vk[7] = {0, 0, d, d, 0, 0, 0};
      r = vr[s - np];
      k = vk[s - np];
    }
    const bool ok = k ? (t.ndim == 2 && t.shape[0] == r && t.shape[1] == k) : (t.ndim == 1 && t.shape[0] == r);
    if (!ok) return fail(ctx, VLA_E_WEIGHTS, "tensor '%s' has the wrong shape", t.name);
    slot[s] = &t;
  }
  return VLA_OK;
}

int require_slots(vla_ctx* ctx, const std::vector<const vla_tensor*>& slot, int first, int last, bool present) {
  for (int s = first; s < last; ++s)
    if ((slot[s] != nullptr) != present)
      return fail(ctx, VLA_E_WEIGHTS, present ? "missing tensor '%s'" : "tensor '%s' does not belong in this call",
                  slot_name(ctx->cfg, s).c_str());
  return VLA_OK;
}

// Enqueues the copy / re-encoding of one tensor into its place in the arena.
void write_slot(vla_ctx* ctx, int s, const vla_tensor* t, hipStream_t st) {
  const vla_config& c = ctx->cfg;
  const ArenaLayout& a = ctx->al;
  const int64_t d = c.d_model, f = c.d_ffn, V = c.vocab, A = c.n_action_bins;
  const bool bf = c.dtype == VLA_BF16;
  const int np = policy_slots(c);
  const bool two = s >= 3 && s < np && two_term_layer(c, (s - 3) / 9);   // tensor of a two-term layer
  auto to_f32 = [&](size_t off, size_t n) {
    if (bf) convert_copy<bf16>((const bf16*)t->dev_ptr, at<float>(ctx->arena, off), n, st);
    else convert_copy<float>((const float*)t->dev_ptr, at<float>(ctx->arena, off), n, st);
  };
  // off8: where the 8-bit copy of the same (fused) matrix starts, used when its low terms are 8-bit
  auto matrix = [&](size_t off, size_t off8, int64_t rows, int64_t K, int64_t row0, int mode) {
    if (bf) {
      pack_weight_f16((const bf16*)t->dev_ptr, (int)rows, (int)K, at<f16>(ctx->arena, off),
                      lo8(two, (int)K) ? at<unsigned char>(ctx->arena, off8) : nullptr, (int)row0, mode,
                      at<int32_t>(ctx->work, ctx->wl.range_flag), st);
    } else {
      const int64_t r0 = mode == 2 ? rows : row0;   // float32 path keeps [gate rows | up rows]
      plain_copy<float>((const float*)t->dev_ptr, at<float>(ctx->arena, off) + r0 * K, (size_t)(rows * K), st);
    }
  };
  auto raw = [&](const void* src, size_t off, size_t n) {
    if (bf) plain_copy<bf16>((const bf16*)src, at<bf16>(ctx->arena, off), n, st);
    else plain_copy<float>((const float*)src, at<float>(ctx->arena, off), n, st);
  };
  if (s == 0) raw(t->dev_ptr, a.embed, (size_t)(V * d));
  else if (s == 1) to_f32(a.g_final, d);
  else if (s == 2) {
    const size_t skip = t->shape[0] == A ? 0 : (size_t)((V - A) * d) * elem_size(c.dtype);
    raw((const char*)t->dev_ptr + skip, a.head, (size_t)(A * d));
  } else if (s < np) {
    const LayerW& lw = a.layers[(s - 3) / 9];
    switch ((s - 3) % 9) {
      case 0: to_f32(lw.g_attn, d); break;
      case 1: matrix(lw.w_qkv, lw.w_qkv8, d, d, 0, 0); break;
      case 2: matrix(lw.w_qkv, lw.w_qkv8, d, d, d, 0); break;
      case 3: matrix(lw.w_qkv, lw.w_qkv8, d, d, 2 * d, 0); break;
      case 4: matrix(lw.w_o, lw.w_o8, d, d, 0, 0); break;
      case 5: to_f32(lw.g_ffn, d); break;
      case 6: matrix(lw.w_gu, lw.w_gu8, f, d, 0, 1); break;
      case 7: matrix(lw.w_gu, lw.w_gu8, f, d, 0, 2); break;
      default: matrix(lw.w_down, lw.w_down8, d, f, 0, 0); break;
    }
  } else {
    switch (s - np) {
      case 0: to_f32(a.v_attn_w, d); break;
      case 1: to_f32(a.v_attn_b, 1); break;
      case 2: raw(t->dev_ptr, a.v_step_emb, (size_t)c.value_max_steps * d); break;
      case 3: raw(t->dev_ptr, a.v_w1, (size_t)(d * d)); break;
      case 4: to_f32(a.v_b1, d); break;
      case 5: to_f32(a.v_w2, d); break;
      default: to_f32(a.v_b2, 1); break;
    }
  }
}

// A whole-set load outside an update: ordered after the compute calls enqueued so far and before the
// ones that follow, on whatever streams those run.
int load_slots(vla_ctx* ctx, const std::vector<const vla_tensor*>& slot, bool whole_policy_set, hipStream_t st) {
  if (ctx->have_work) HIP_TRY(ctx, hipStreamWaitEvent(st, ctx->ev_work, 0));
  int rc = VLA_OK;
  if (whole_policy_set && (rc = range_check_begin(ctx, st))) return rc;   // every matrix is rewritten: start clean
  for (size_t s = 0; s < slot.size(); ++s)
    if (slot[s]) write_slot(ctx, (int)s, slot[s], st);
  HIP_TRY(ctx, hipGetLastError());
  if ((rc = range_check_end(ctx, st))) return rc;
  HIP_TRY(ctx, hipEventRecord(ctx->ev_update, st));
  ctx->have_update = true;
  ctx->version += 1;
  ctx->active_B = 0;     // cached keys / values belong to the old weights
  ctx->len.assign(ctx->cfg.max_batch, 0);
  return VLA_OK;
}

int check_loadable(vla_ctx* ctx, const vla_tensor* tensors) {
  if (!tensors) return fail(ctx, VLA_E_NULL, "tensors is NULL");
  if (!ctx->bound) return fail(ctx, VLA_E_STATE, "buffers are not bound (vla_bind_buffers)");
  if (ctx->serving == VLA_UPDATING) return fail(ctx, VLA_E_DRAINING, "an update is open (vla_update_tensors / vla_update_commit)");
  return VLA_OK;
}

}  // namespace

extern "C" {

int vla_load_weights(vla_ctx* ctx, const vla_tensor* tensors, int32_t n_tensors, void* hip_stream) {
  if (!ctx) return VLA_E_NULL;
  int rc = check_loadable(ctx, tensors);
  if (rc) return rc;
  std::vector<const vla_tensor*> slot(all_slots(ctx->cfg), nullptr);
  if ((rc = parse_tensors(ctx, tensors, n_tensors, slot))) return rc;
  if ((rc = require_slots(ctx, slot, 0, policy_slots(ctx->cfg), true))) return rc;
  if ((rc = require_slots(ctx, slot, policy_slots(ctx->cfg), all_slots(ctx->cfg), false))) return rc;
  if ((rc = load_slots(ctx, slot, true, (hipStream_t)hip_stream))) return rc;
  ctx->weights = true;
  return VLA_OK;
}

int vla_load_value_head(vla_ctx* ctx, const vla_tensor* tensors, int32_t n_tensors, void* hip_stream) {
  if (!ctx) return VLA_E_NULL;
  int rc = check_loadable(ctx, tensors);
  if (rc) return rc;
  if (ctx->cfg.value_max_steps <= 0) return fail(ctx, VLA_E_CONFIG, "the context was created without a value head");
  std::vector<const vla_tensor*> slot(all_slots(ctx->cfg), nullptr);
  if ((rc = parse_tensors(ctx, tensors, n_tensors, slot))) return rc;
  if ((rc = require_slots(ctx, slot, 0, policy_slots(ctx->cfg), false))) return rc;
  if ((rc = require_slots(ctx, slot, policy_slots(ctx->cfg), all_slots(ctx->cfg), true))) return rc;
  if ((rc = load_slots(ctx, slot, false, (hipStream_t)hip_stream))) return rc;
  ctx->value_weights = true;
  return VLA_OK;
}

int vla_check_weights(vla_ctx* ctx) {
  if (!ctx) return VLA_E_NULL;
  if (!ctx->bound) return fail(ctx, VLA_E_STATE, "buffers are not bound (vla_bind_buffers)");
  return poll_weight_range(ctx, true);
}

int vla_get_state(const vla_ctx* ctx, int32_t* state, int64_t* version) {
  if (!ctx) return VLA_E_NULL;
  if (state) *state = ctx->serving;
  if (version) *version = ctx->version;
  return VLA_OK;
}

int vla_drain_begin(vla_ctx* ctx) {
  if (!ctx) return VLA_E_NULL;
  if (ctx->serving == VLA_UPDATING) return fail(ctx, VLA_E_DRAINING, "an update is already open");
  ctx->serving = VLA_DRAINING;
  return VLA_OK;
}

int vla_update_begin(vla_ctx* ctx, void* hip_stream) {
  if (!ctx) return VLA_E_NULL;
  if (!ctx->bound) return fail(ctx, VLA_E_STATE, "buffers are not bound (vla_bind_buffers)");
  if (!ctx->weights) return fail(ctx, VLA_E_STATE, "nothing to update: weights were never loaded (vla_load_weights)");
  if (ctx->serving == VLA_UPDATING) return fail(ctx, VLA_E_DRAINING, "an update is already open");
  if (ctx->have_work) HIP_TRY(ctx, hipStreamWaitEvent((hipStream_t)hip_stream, ctx->ev_work, 0));
  ctx->serving = VLA_UPDATING;
  ctx->active_B = 0;     // the batch in flight has been enqueued to its end; its cache dies with the old weights
  ctx->len.assign(ctx->cfg.max_batch, 0);
  return VLA_OK;
}

int vla_update_tensors(vla_ctx* ctx, const vla_tensor* tensors, int32_t n_tensors, void* hip_stream) {
  if (!ctx) return VLA_E_NULL;
  if (!tensors) return fail(ctx, VLA_E_NULL, "tensors is NULL");
  if (ctx->serving != VLA_UPDATING) return fail(ctx, VLA_E_STATE, "no update is open (vla_update_begin)");
  std::vector<const vla_tensor*> slot(all_slots(ctx->cfg), nullptr);
  int rc = parse_tensors(ctx, tensors, n_tensors, slot);
  if (rc) return rc;
  if (!ctx->value_weights)     // a first value head must arrive whole
    for (int s = policy_slots(ctx->cfg); s < all_slots(ctx->cfg); ++s)
      if (slot[s]) return fail(ctx, VLA_E_STATE, "'%s': load the value head once (vla_load_value_head) before updating it", slot_name(ctx->cfg, s).c_str());
  for (size_t s = 0; s < slot.size(); ++s)
    if (slot[s]) write_slot(ctx, (int)s, slot[s], (hipStream_t)hip_stream);
  HIP_TRY(ctx, hipGetLastError());
  return VLA_OK;
}

int vla_update_commit(vla_ctx* ctx, void* hip_stream, int64_t* version_out) {
  if (!ctx) return VLA_E_NULL;
  if (ctx->serving != VLA_UPDATING) return fail(ctx, VLA_E_STATE, "no update is open (vla_update_begin)");
  int rc = range_check_end(ctx, (hipStream_t)hip_stream);
  if (rc) return rc;
  HIP_TRY(ctx, hipEventRecord(ctx->ev_update, (hipStream_t)hip_stream));
  ctx->have_update = true;
  ctx->version += 1;
  ctx->serving = VLA_ACCEPTING;
  if (version_out) *version_out = ctx->version;
  return VLA_OK;
}

int vla_prefill(vla_ctx* ctx, int32_t B, const void* patch_emb, const int32_t* cu_patch, const int32_t* instr_ids,
                const int32_t* cu_instr, float* logits_out, void* hip_stream) {
  if (!ctx) return VLA_E_NULL;
  int rc = check_ready(ctx);
  if (rc) return rc;
  if ((rc = check_serving(ctx, true))) return rc;
  int64_t T = 0;
  rc = check_prefill(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, 0, &T);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  if ((rc = enter_compute(ctx, st))) return rc;
  const int A = ctx->cfg.n_action_bins;
  rc = ctx->cfg.dtype == VLA_BF16 ? do_prefill<bf16>(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, T, logits_out, A, st)
                                  : do_prefill<float>(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, T, logits_out, A, st);
  if (rc) return rc;
  return leave_compute(ctx, st);
}

int vla_decode_step(vla_ctx* ctx, int32_t B, const int32_t* token_ids, float* logits_out, void* hip_stream) {
  if (!ctx) return VLA_E_NULL;
  int rc = check_ready(ctx);
  if (rc) return rc;
  if ((rc = check_serving(ctx, false))) return rc;
  if (!token_ids) return fail(ctx, VLA_E_NULL, "token_ids is NULL");
  rc = check_decode(ctx, B, 1);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  if ((rc = enter_compute(ctx, st))) return rc;
  const int A = ctx->cfg.n_action_bins;
  rc = ctx->cfg.dtype == VLA_BF16 ? do_decode<bf16>(ctx, B, token_ids, logits_out, A, st)
                                  : do_decode<float>(ctx, B, token_ids, logits_out, A, st);
  if (rc) return rc;
  return leave_compute(ctx, st);
}

int vla_decode_step_static(vla_ctx* ctx, int32_t B, const int32_t* token_ids, float* logits_out, void* hip_stream) {
  if (!ctx) return VLA_E_NULL;
  int rc = check_ready(ctx);
  if (rc) return rc;
  if ((rc = check_serving(ctx, false))) return rc;
  if (!token_ids) return fail(ctx, VLA_E_NULL, "token_ids is NULL");
  if ((rc = check_decode(ctx, B, 1))) return rc;
  const vla_config& c = ctx->cfg;
  // staging the step's GEMMs need: the split-K partial planes of the 16-bit path (rows of one chunk), or the
  // plain GEMM output of the float32 path
  const size_t widest = 3 * (size_t)c.d_model > 2 * (size_t)c.d_ffn ? 3 * (size_t)c.d_model : 2 * (size_t)c.d_ffn;
  const size_t rows = c.dtype == VLA_BF16 ? (size_t)kMaxKSplit * B : (size_t)B;
  const size_t need = rows * widest * sizeof(float);
  if (need > kStaticScratchBytes)
    return fail(ctx, VLA_E_CAPACITY, "vla_decode_step_static: batch %d of this model needs %zu bytes of staging, the static "
                "array holds %zu (use vla_decode_step)", B, need, kStaticScratchBytes);
  void* sp = nullptr;
  HIP_TRY(ctx, static_scratch(&sp));
  hipStream_t st = (hipStream_t)hip_stream;
  if ((rc = enter_compute(ctx, st))) return rc;
  const int A = c.n_action_bins;
  ctx->part_override = (float*)sp;       // every element read from it in this step is written earlier in this step
  rc = c.dtype == VLA_BF16 ? do_decode<bf16>(ctx, B, token_ids, logits_out, A, st)
                           : do_decode<float>(ctx, B, token_ids, logits_out, A, st);
  ctx->part_override = nullptr;
  if (rc) return rc;
  return leave_compute(ctx, st);
}

int vla_prefill_slots(vla_ctx* ctx, int32_t n, const int32_t* slot_ids, const void* patch_emb, const int32_t* cu_patch,
                      const int32_t* instr_ids, const int32_t* cu_instr, float* logits_out, void* hip_stream) {
  if (!ctx) return VLA_E_NULL;
  int rc = check_ready(ctx);
  if (rc) return rc;
  if ((rc = check_serving(ctx, true))) return rc;
  if ((rc = check_slots(ctx, n, slot_ids))) return rc;
  int64_t T = 0;
  if ((rc = check_prefill(ctx, n, patch_emb, cu_patch, instr_ids, cu_instr, 0, &T))) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  if ((rc = enter_compute(ctx, st))) return rc;
  const int A = ctx->cfg.n_action_bins;
  rc = ctx->cfg.dtype == VLA_BF16
           ? do_prefill<bf16>(ctx, n, patch_emb, cu_patch, instr_ids, cu_instr, T, logits_out, A, st, nullptr, 0, slot_ids)
           : do_prefill<float>(ctx, n, patch_emb, cu_patch, instr_ids, cu_instr, T, logits_out, A, st, nullptr, 0, slot_ids);
  if (rc) return rc;
  return leave_compute(ctx, st);
}

int vla_decode_slots(vla_ctx* ctx, int32_t n, const int32_t* slot_ids, const int32_t* token_ids, float* logits_out,
                     void* hip_stream) {
  if (!ctx) return VLA_E_NULL;
  int rc = check_ready(ctx);
  if (rc) return rc;
  if ((rc = check_serving(ctx, false))) return rc;
  if (!token_ids) return fail(ctx, VLA_E_NULL, "token_ids is NULL");
  if ((rc = check_slots(ctx, n, slot_ids))) return rc;
  if ((int)ctx->len.size() < ctx->cfg.max_batch) ctx->len.resize(ctx->cfg.max_batch, 0);
  for (int i = 0; i < n; ++i) {
    const int len = ctx->len[slot_ids[i]];
    if (len == 0) return fail(ctx, VLA_E_STATE, "slot %d holds no sequence (prefill it first)", slot_ids[i]);
    if (len + 1 > ctx->cfg.max_seq)
      return fail(ctx, VLA_E_CAPACITY, "slot %d is full (%d of %d positions)", slot_ids[i], len, ctx->cfg.max_seq);
  }
  hipStream_t st = (hipStream_t)hip_stream;
  if ((rc = enter_compute(ctx, st))) return rc;
  const int A = ctx->cfg.n_action_bins;
  rc = ctx->cfg.dtype == VLA_BF16 ? do_decode<bf16>(ctx, n, token_ids, logits_out, A, st, slot_ids)
                                  : do_decode<float>(ctx, n, token_ids, logits_out, A, st, slot_ids);
  if (rc) return rc;
  return leave_compute(ctx, st);
}

int vla_release_slots(vla_ctx* ctx, int32_t n, const int32_t* slot_ids) {
  if (!ctx) return VLA_E_NULL;
  int rc = check_slots(ctx, n, slot_ids);
  if (rc) return rc;
  if ((int)ctx->len.size() < ctx->cfg.max_batch) ctx->len.resize(ctx->cfg.max_batch, 0);
  for (int i = 0; i < n; ++i) ctx->len[slot_ids[i]] = 0;
  ctx->active_B = 0;
  return VLA_OK;
}

int vla_select(vla_ctx* ctx, int32_t B, const float* logits, float temperature, const float* gumbel, int32_t k,
               int32_t n_tokens, const float* act_scale, const float* act_offset, int32_t action_dim,
               int32_t* tokens_out, float* logp_out, float* actions_out, int32_t out_stride, int32_t* next_ids_out,
               void* hip_stream) {
  if (!ctx) return VLA_E_NULL;
  if (!logits || !tokens_out || !logp_out || !actions_out) return fail(ctx, VLA_E_NULL, "a required pointer is NULL");
  if (B <= 0 || k < 0 || n_tokens <= 0 || k >= n_tokens || out_stride < n_tokens || action_dim < 0 || !(temperature >= 0.f))
    return fail(ctx, VLA_E_SHAPE, "bad selection arguments");
  const vla_config& c = ctx->cfg;
  ProfScope ps(ctx, FAM_HEAD, (hipStream_t)hip_stream);
  select_tokens(logits, c.n_action_bins, B, c.n_action_bins, temperature, gumbel, k, n_tokens, act_scale, act_offset,
                action_dim, tokens_out, logp_out, actions_out, out_stride, next_ids_out, c.vocab - c.n_action_bins,
                (hipStream_t)hip_stream);
  HIP_TRY(ctx, hipGetLastError());
  return VLA_OK;
}

static int policy_step_impl(vla_ctx* ctx, int32_t B, const void* patch_emb, const int32_t* cu_patch,
                            const int32_t* instr_ids, const int32_t* cu_instr, int32_t n_tokens, float temperature,
                            const float* gumbel, const float* act_scale, const float* act_offset, int32_t action_dim,
                            const int32_t* step_t, int32_t* tokens_out, float* logp_out, float* actions_out,
                            float* logits_out, float* values_out, bool with_value, void* hip_stream) {
  if (!ctx) return VLA_E_NULL;
  int rc = check_ready(ctx);
  if (rc) return rc;
  if ((rc = check_serving(ctx, true))) return rc;
  if (!tokens_out || !logp_out || !actions_out) return fail(ctx, VLA_E_NULL, "an output pointer is NULL");
  if (n_tokens <= 0) return fail(ctx, VLA_E_SHAPE, "n_tokens must be positive");
  if (!(temperature >= 0.f)) return fail(ctx, VLA_E_SHAPE, "temperature must be >= 0");
  if (action_dim < 0) return fail(ctx, VLA_E_SHAPE, "action_dim must be >= 0");
  if (with_value) {
    if (ctx->cfg.value_max_steps <= 0) return fail(ctx, VLA_E_CONFIG, "the context was created without a value head");
    if (!ctx->value_weights) return fail(ctx, VLA_E_STATE, "value head weights are not loaded (vla_load_value_head)");
    if (!step_t || !values_out) return fail(ctx, VLA_E_NULL, "step_t / values_out is NULL");
  }
  int64_t T = 0;
  rc = check_prefill(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, n_tokens, &T);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  if ((rc = enter_compute(ctx, st))) return rc;
  const vla_config& c = ctx->cfg;
  const int A = c.n_action_bins, id0 = c.vocab - A;
  int32_t* cur = at<int32_t>(ctx->work, ctx->wl.cur_ids);
  float* own = at<float>(ctx->work, ctx->wl.logits);
  const bool bf = c.dtype == VLA_BF16;
  for (int k = 0; k < n_tokens; ++k) {
    float* lg = logits_out ? logits_out + (size_t)k * A : own;
    const int ld = logits_out ? n_tokens * A : A;
    if (k == 0)
      rc = bf ? do_prefill<bf16>(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, T, lg, ld, st)
              : do_prefill<float>(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, T, lg, ld, st);
    else
      rc = bf ? do_decode<bf16>(ctx, B, cur, lg, ld, st) : do_decode<float>(ctx, B, cur, lg, ld, st);
    if (rc) return rc;
    if (with_value) run_value_accumulate(ctx, B, k == 0 ? at<int32_t>(ctx->work, ctx->wl.last_row) : nullptr, k == 0, st);
    ProfScope ps(ctx, FAM_HEAD, st);
    select_tokens(lg, ld, B, A, temperature, gumbel, k, n_tokens, act_scale, act_offset, action_dim, tokens_out,
                  logp_out, actions_out, n_tokens, cur, id0, st);
  }
  if (with_value) {
    ProfScope ps(ctx, FAM_HEAD, st);
    const ArenaLayout& a = ctx->al;
    const WorkLayout& w = ctx->wl;
    if (bf)
      value_finish<bf16>(at<float>(ctx->work, w.vz), at<float>(ctx->work, w.vml), at<bf16>(ctx->arena, a.v_step_emb),
                         c.value_max_steps, step_t, at<bf16>(ctx->arena, a.v_w1), at<float>(ctx->arena, a.v_b1),
                         at<float>(ctx->arena, a.v_w2), at<float>(ctx->arena, a.v_b2), B, c.d_model,
                         at<float>(ctx->work, w.vu), at<float>(ctx->work, w.vh), values_out, st);
    else
      value_finish<float>(at<float>(ctx->work, w.vz), at<float>(ctx->work, w.vml), at<float>(ctx->arena, a.v_step_emb),
                          c.value_max_steps, step_t, at<float>(ctx->arena, a.v_w1), at<float>(ctx->arena, a.v_b1),
                          at<float>(ctx->arena, a.v_w2), at<float>(ctx->arena, a.v_b2), B, c.d_model,
                          at<float>(ctx->work, w.vu), at<float>(ctx->work, w.vh), values_out, st);
  }
  HIP_TRY(ctx, hipGetLastError());
  return leave_compute(ctx, st);
}

int vla_policy_step(vla_ctx* ctx, int32_t B, const void* patch_emb, const int32_t* cu_patch, const int32_t* instr_ids,
                    const int32_t* cu_instr, int32_t n_tokens, float temperature, const float* gumbel,
                    const float* act_scale, const float* act_offset, int32_t action_dim, int32_t* tokens_out,
                    float* logp_out, float* actions_out, float* logits_out, void* hip_stream) {
  return policy_step_impl(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, n_tokens, temperature, gumbel, act_scale,
                          act_offset, action_dim, nullptr, tokens_out, logp_out, actions_out, logits_out, nullptr,
                          false, hip_stream);
}

int vla_policy_step_value(vla_ctx* ctx, int32_t B, const void* patch_emb, const int32_t* cu_patch,
                          const int32_t* instr_ids, const int32_t* cu_instr, int32_t n_tokens, float temperature,
                          const float* gumbel, const float* act_scale, const float* act_offset, int32_t action_dim,
                          const int32_t* step_t, int32_t* tokens_out, float* logp_out, float* actions_out,
                          float* logits_out, float* values_out, void* hip_stream) {
  return policy_step_impl(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, n_tokens, temperature, gumbel, act_scale,
                          act_offset, action_dim, step_t, tokens_out, logp_out, actions_out, logits_out, values_out,
                          true, hip_stream);
}

int vla_policy_step_parallel(vla_ctx* ctx, int32_t B, const void* patch_emb, const int32_t* cu_patch,
                             const int32_t* instr_ids, const int32_t* cu_instr, int32_t n_tokens,
                             int32_t placeholder_id, float temperature, const float* gumbel, const float* act_scale,
                             const float* act_offset, int32_t action_dim, int32_t* tokens_out, float* logp_out,
                             float* actions_out, float* logits_out, void* hip_stream) {
  if (!ctx) return VLA_E_NULL;
  int rc = check_ready(ctx);
  if (rc) return rc;
  if ((rc = check_serving(ctx, true))) return rc;
  if (!tokens_out || !logp_out || !actions_out) return fail(ctx, VLA_E_NULL, "an output pointer is NULL");
  if (!(temperature >= 0.f)) return fail(ctx, VLA_E_SHAPE, "temperature must be >= 0");
  if (action_dim < 0) return fail(ctx, VLA_E_SHAPE, "action_dim must be >= 0");
  const vla_config& c = ctx->cfg;
  if (placeholder_id < 0 || placeholder_id >= c.vocab) return fail(ctx, VLA_E_SHAPE, "placeholder_id outside the vocabulary");
  int64_t T = 0;
  if ((rc = check_chunk(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, n_tokens, &T))) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  if ((rc = enter_compute(ctx, st))) return rc;
  const int A = c.n_action_bins, K = n_tokens;
  float* lg = logits_out ? logits_out : at<float>(ctx->work, ctx->wl.chunk_logits);
  rc = c.dtype == VLA_BF16
           ? do_chunk<bf16>(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, T, K, nullptr, placeholder_id, lg, st)
           : do_chunk<float>(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, T, K, nullptr, placeholder_id, lg, st);
  if (rc) return rc;
  {
    ProfScope ps(ctx, FAM_HEAD, st);
    for (int k = 0; k < K; ++k)
      select_tokens(lg + (size_t)k * A, K * A, B, A, temperature, gumbel, k, K, act_scale, act_offset, action_dim,
                    tokens_out, logp_out, actions_out, K, nullptr, c.vocab - A, st);
  }
  HIP_TRY(ctx, hipGetLastError());
  return leave_compute(ctx, st);
}

int vla_score_tokens(vla_ctx* ctx, int32_t B, const void* patch_emb, const int32_t* cu_patch, const int32_t* instr_ids,
                     const int32_t* cu_instr, int32_t n_tokens, const int32_t* tokens, int32_t placeholder_id,
                     float temperature, const float* mu_logp, float sigma, float* logp_out, float* ratio_out,
                     float* weight_out, float* logits_out, void* hip_stream) {
  if (!ctx) return VLA_E_NULL;
  int rc = check_ready(ctx);
  if (rc) return rc;
  if ((rc = check_serving(ctx, true))) return rc;
  if (!tokens || !logp_out) return fail(ctx, VLA_E_NULL, "tokens / logp_out is NULL");
  if (!(temperature >= 0.f)) return fail(ctx, VLA_E_SHAPE, "temperature must be >= 0");
  if ((ratio_out || weight_out) && !mu_logp) return fail(ctx, VLA_E_NULL, "ratio / weight need mu_logp");
  if (mu_logp && weight_out && !(sigma > 0.f)) return fail(ctx, VLA_E_SHAPE, "sigma must be positive");
  const vla_config& c = ctx->cfg;
  if (placeholder_id >= c.vocab) return fail(ctx, VLA_E_SHAPE, "placeholder_id outside the vocabulary");
  int64_t T = 0;
  if ((rc = check_chunk(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, n_tokens, &T))) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  if ((rc = enter_compute(ctx, st))) return rc;
  const int A = c.n_action_bins, K = n_tokens;
  float* lg = logits_out ? logits_out : at<float>(ctx->work, ctx->wl.chunk_logits);
  const int32_t* stored = placeholder_id < 0 ? tokens : nullptr;
  rc = c.dtype == VLA_BF16
           ? do_chunk<bf16>(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, T, K, stored, placeholder_id, lg, st)
           : do_chunk<float>(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, T, K, stored, placeholder_id, lg, st);
  if (rc) return rc;
  {
    ProfScope ps(ctx, FAM_HEAD, st);
    score_rows(lg, B * K, A, temperature, tokens, mu_logp, sigma, logp_out, ratio_out, weight_out, st);
  }
  HIP_TRY(ctx, hipGetLastError());
  return leave_compute(ctx, st);
}

int vla_probe(vla_ctx* ctx, int32_t kind, double* value_out, void* hip_stream) {
  if (!ctx) return VLA_E_NULL;
  if (!value_out) return fail(ctx, VLA_E_NULL, "value_out is NULL");
  if (!ctx->bound || !ctx->weights) return fail(ctx, VLA_E_STATE, "the probes read the loaded weight arena");
  if (ctx->cfg.dtype != VLA_BF16) return fail(ctx, VLA_E_CONFIG, "the probes are for the 16-bit path");
  if (kind != 0 && kind != 1) return fail(ctx, VLA_E_SHAPE, "kind must be 0 (MFMA loop) or 1 (streaming read)");
  hipStream_t st = (hipStream_t)hip_stream;
  // layer 0's fused gate/up matrix: fragment-ordered half-precision weights
  const vla_config& c = ctx->cfg;
  const f16* w = at<f16>(ctx->arena, ctx->al.layers[0].w_gu);
  const size_t w_bytes = (size_t)2 * c.d_ffn * c.d_model * sizeof(f16);
  const size_t bytes = kind == 1 ? ctx->al.total - ctx->al.layers[0].w_qkv : 0;   // all layer matrices and gains
  float* sink = at<float>(ctx->work, ctx->wl.logits);
  hipEvent_t e0, e1;
  HIP_TRY(ctx, hipEventCreate(&e0));
  HIP_TRY(ctx, hipEventCreate(&e1));
  const int n_wg = 512, iters = 8192, reps = 3;
  float best = 1e30f;
  for (int r = 0; r < reps + 1; ++r) {     // first run warms up
    HIP_TRY(ctx, hipEventRecord(e0, st));
    if (kind == 0) probe_mfma(w, w_bytes / 1024, n_wg, iters, sink, st);
    else probe_stream(at<char>(ctx->arena, ctx->al.layers[0].w_qkv), bytes, 4096, (unsigned*)sink, st);
    HIP_TRY(ctx, hipEventRecord(e1, st));
    HIP_TRY(ctx, hipEventSynchronize(e1));
    float ms = 0.f;
    HIP_TRY(ctx, hipEventElapsedTime(&ms, e0, e1));
    if (r > 0 && ms < best) best = ms;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  HIP_TRY(ctx, hipGetLastError());
  if (kind == 0) *value_out = (double)n_wg * 4 * iters * 8 * 32768.0 / (best * 1e-3) / 1e12;   // TFLOP/s
  else *value_out = (double)bytes / (best * 1e-3) / 1e9;                                        // GB/s
  return VLA_OK;
}

int vla_prof_enable(vla_ctx* ctx, int32_t mask) {
  if (!ctx) return VLA_E_NULL;
  for (auto& v : ctx->prof) {
    for (auto& p : v) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
    v.clear();
  }
  ctx->prof_mask = (unsigned)mask;
  return VLA_OK;
}

int vla_prof_count(void) { return FAM_COUNT; }

int vla_prof_read(vla_ctx* ctx, int32_t i, const char** name, int64_t* launches, double* total_ms) {
  if (!ctx) return VLA_E_NULL;
  if (i < 0 || i >= FAM_COUNT) return fail(ctx, VLA_E_SHAPE, "family index out of range");
  double tot = 0.0;
  for (auto& p : ctx->prof[i]) {
    HIP_TRY(ctx, hipEventSynchronize(p.b));
    float ms = 0.f;
    HIP_TRY(ctx, hipEventElapsedTime(&ms, p.a, p.b));
    tot += ms;
  }
  if (name) *name = kFamilyNames[i];
  if (launches) *launches = (int64_t)ctx->prof[i].size();
  if (total_ms) *total_ms = tot;
  return VLA_OK;
}

}  // extern "C"
