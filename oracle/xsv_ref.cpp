// xsv_ref — CPU oracle for the XStreamVGGT per-frame streaming step.
//
// TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library, its Python binding)
// may include, link, import or call this file; only tests, the smoke check and the benchmark's
// CPU-baseline leg do.  It shares no code with the HIP kernels.
//
// Plain, slow, single-precision C++ written from the paper's equations, in the paper's order:
//   Sec. 3.1  (cache definition, temporal attention over [cache ; current frame])
//   Sec. 3.2  (pooled-query importance score, top-k of the prunable middle, retained index set)
//   Sec. 3.3  (asymmetric uniform quantization; keys per channel, values per token; dequantize
//              at attention time)
// No blocking, fusion or reordering: every loop below is the definition written out.
// Build: g++ -O2 -ffp-contract=off -fopenmp -shared -fPIC.  OpenMP is used over heads / rows only
// (independent outputs), never inside a reduction, so results do not depend on the thread count.
//
// Precision: fp32 throughout, because the quantizer's integer decisions (codes, zero points) are
// defined on fp32 scale factors and both sides must take them in the same precision.  Inputs and
// the dequantized cache view are bf16 (round-to-nearest-even).
//
// Parity pins live in tests/ (markers "not gpu").  Unpinned against the authors' own outputs:
// the paper prints no worked example and ships no code; the readings taken where it is silent are
// listed next to each function.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <numeric>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

// ---- bf16 <-> fp32 -------------------------------------------------------------------------
inline float bf16_to_f32(uint16_t b) {
  uint32_t u = static_cast<uint32_t>(b) << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

inline uint16_t f32_to_bf16(float f) {  // round to nearest, ties to even
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x0040u);  // NaN
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  return static_cast<uint16_t>(u >> 16);
}

inline float round_bf16(float f) { return bf16_to_f32(f32_to_bf16(f)); }

// ---- Sec. 3.3, quantizer of one group ---------------------------------------------------------
// s = (x_max - x_min) / (2^b - 1),  z = round(-x_min / s),  code = clamp(round(x / s) + z, 0, 2^b-1).
// Readings where the paper is silent: round = nearest, ties to even; a constant group (s == 0)
// takes s = 1; z is an integer-valued float and is not clamped.
struct GroupParams {
  float s, z;
};

inline GroupParams group_params(float x_min, float x_max, int bits) {
  const float levels = static_cast<float>((1 << bits) - 1);
  float s = (x_max - x_min) / levels;
  if (s == 0.0f) s = 1.0f;
  float z = std::nearbyintf(-x_min / s);
  return {s, z};
}

inline uint8_t quantize_one(float x, GroupParams p, int bits) {
  const float hi = static_cast<float>((1 << bits) - 1);
  float q = std::nearbyintf(x / p.s) + p.z;
  q = std::min(std::max(q, 0.0f), hi);
  return static_cast<uint8_t>(q);
}

// Dequantized view used by every consumer (attention, scoring, re-quantization):
// (code - z) * s, rounded to bf16.
inline float dequantize_one(uint8_t code, float s, float z) {
  return round_bf16((static_cast<float>(code) - z) * s);
}

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// memcpy that tolerates empty ranges (an empty cache has no storage to point at)
inline void copy_bytes(void* dst, const void* src, size_t n) {
  if (n != 0) std::memcpy(dst, src, n);
}

}  // namespace

extern "C" {

// ------------------------------------------------------------------------------------------------
// Sec. 3.3: keys are quantized per channel.  One group = one (head, channel) over G consecutive
// cached tokens; the last group of a cache whose length is not a multiple of G is short and is
// quantized on its own.
//   k      [H][T][d] bf16
//   codes  [H][T][d] one code per byte
//   scale, zero [H][ceil(T/G)][d]
void xsv_ref_quantize_k(const uint16_t* k, int H, int T, int d, int bits, int G, uint8_t* codes,
                        float* scale, float* zero) {
  const int n_groups = ceil_div(T, G);
#pragma omp parallel for schedule(static)
  for (int h = 0; h < H; ++h) {
    for (int u = 0; u < n_groups; ++u) {
      const int t0 = u * G, t1 = std::min(T, t0 + G);
      for (int c = 0; c < d; ++c) {
        float lo = bf16_to_f32(k[(static_cast<size_t>(h) * T + t0) * d + c]);
        float hi = lo;
        for (int t = t0; t < t1; ++t) {
          float x = bf16_to_f32(k[(static_cast<size_t>(h) * T + t) * d + c]);
          lo = std::min(lo, x);
          hi = std::max(hi, x);
        }
        GroupParams p = group_params(lo, hi, bits);
        scale[(static_cast<size_t>(h) * n_groups + u) * d + c] = p.s;
        zero[(static_cast<size_t>(h) * n_groups + u) * d + c] = p.z;
        for (int t = t0; t < t1; ++t) {
          size_t i = (static_cast<size_t>(h) * T + t) * d + c;
          codes[i] = quantize_one(bf16_to_f32(k[i]), p, bits);
        }
      }
    }
  }
}

// Sec. 3.3: values are quantized per token.  One group = one (head, token) over G consecutive
// channels of that head (d / G groups per token).
//   v      [H][T][d] bf16
//   codes  [H][T][d]
//   scale, zero [H][T][d/G]
void xsv_ref_quantize_v(const uint16_t* v, int H, int T, int d, int bits, int G, uint8_t* codes,
                        float* scale, float* zero) {
  const int n_groups = d / G;
#pragma omp parallel for schedule(static)
  for (int h = 0; h < H; ++h) {
    for (int t = 0; t < T; ++t) {
      for (int u = 0; u < n_groups; ++u) {
        const size_t base = (static_cast<size_t>(h) * T + t) * d + static_cast<size_t>(u) * G;
        float lo = bf16_to_f32(v[base]);
        float hi = lo;
        for (int c = 0; c < G; ++c) {
          float x = bf16_to_f32(v[base + c]);
          lo = std::min(lo, x);
          hi = std::max(hi, x);
        }
        GroupParams p = group_params(lo, hi, bits);
        scale[(static_cast<size_t>(h) * T + t) * n_groups + u] = p.s;
        zero[(static_cast<size_t>(h) * T + t) * n_groups + u] = p.z;
        for (int c = 0; c < G; ++c) codes[base + c] = quantize_one(bf16_to_f32(v[base + c]), p, bits);
      }
    }
  }
}

// Sec. 3.3, dequantization operators (per channel for keys, per token for values) → bf16 view.
void xsv_ref_dequantize_k(const uint8_t* codes, const float* scale, const float* zero, int H, int T,
                          int d, int G, uint16_t* out) {
  const int n_groups = ceil_div(T, G);
  for (int h = 0; h < H; ++h)
    for (int t = 0; t < T; ++t)
      for (int c = 0; c < d; ++c) {
        size_t i = (static_cast<size_t>(h) * T + t) * d + c;
        size_t g = (static_cast<size_t>(h) * n_groups + t / G) * d + c;
        out[i] = f32_to_bf16(dequantize_one(codes[i], scale[g], zero[g]));
      }
}

void xsv_ref_dequantize_v(const uint8_t* codes, const float* scale, const float* zero, int H, int T,
                          int d, int G, uint16_t* out) {
  const int n_groups = d / G;
  for (int h = 0; h < H; ++h)
    for (int t = 0; t < T; ++t)
      for (int c = 0; c < d; ++c) {
        size_t i = (static_cast<size_t>(h) * T + t) * d + c;
        size_t g = (static_cast<size_t>(h) * T + t) * n_groups + c / G;
        out[i] = f32_to_bf16(dequantize_one(codes[i], scale[g], zero[g]));
      }
}

// ------------------------------------------------------------------------------------------------
// Sec. 3.1, temporal attention of the current frame's queries over [cache ; current frame].
// Inside one streaming step nothing is masked: every key belongs to a frame <= t.
//   q [H][n][d], k, v [H][Tk][d] bf16;  rows: n_rows query indices (NULL → all n rows, n_rows = n)
//   out [H][n_rows][d] fp32:  softmax_j(scale * q·k_j) · v, logits and sums in ascending j / c.
void xsv_ref_attend(const uint16_t* q, const uint16_t* k, const uint16_t* v, int H, int n, int Tk,
                    int d, float scale, const int32_t* rows, int n_rows, float* out) {
  if (rows == nullptr) n_rows = n;
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
  for (int h = 0; h < H; ++h) {
    for (int r = 0; r < n_rows; ++r) {
      const int i = rows ? rows[r] : r;
      std::vector<float> logit(Tk);
      const uint16_t* qi = q + (static_cast<size_t>(h) * n + i) * d;
      float m = -INFINITY;
      for (int j = 0; j < Tk; ++j) {
        const uint16_t* kj = k + (static_cast<size_t>(h) * Tk + j) * d;
        float acc = 0.0f;
        for (int c = 0; c < d; ++c) acc += bf16_to_f32(qi[c]) * bf16_to_f32(kj[c]);
        logit[j] = scale * acc;
        m = std::max(m, logit[j]);
      }
      std::vector<float> o(d, 0.0f);
      float denom = 0.0f;
      for (int j = 0; j < Tk; ++j) {
        float p = std::exp(logit[j] - m);
        denom += p;
        const uint16_t* vj = v + (static_cast<size_t>(h) * Tk + j) * d;
        for (int c = 0; c < d; ++c) o[c] += p * bf16_to_f32(vj[c]);
      }
      float* dst = out + (static_cast<size_t>(h) * n_rows + r) * d;
      for (int c = 0; c < d; ++c) dst[c] = o[c] / denom;
    }
  }
}

// Checker beneath the streamed attention: ONE pass of frame-causal attention over a whole stream
// (Sec. 3.1: a query of frame f sees every token of frames <= f, none of later frames).
//   q, k, v [H][F*n][d] bf16 (frame-major), out [H][F*n][d] fp32.
void xsv_ref_block_causal_attention(const uint16_t* q, const uint16_t* k, const uint16_t* v, int H,
                                    int F, int n, int d, float scale, float* out) {
  const int T = F * n;
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
  for (int h = 0; h < H; ++h) {
    for (int i = 0; i < T; ++i) {
      const int visible = (i / n + 1) * n;  // tokens of frames 0..frame(i)
      std::vector<float> logit(visible);
      float m = -INFINITY;
      for (int j = 0; j < visible; ++j) {
        float acc = 0.0f;
        for (int c = 0; c < d; ++c)
          acc += bf16_to_f32(q[(static_cast<size_t>(h) * T + i) * d + c]) *
                 bf16_to_f32(k[(static_cast<size_t>(h) * T + j) * d + c]);
        logit[j] = scale * acc;
        m = std::max(m, logit[j]);
      }
      std::vector<float> o(d, 0.0f);
      float denom = 0.0f;
      for (int j = 0; j < visible; ++j) {
        float p = std::exp(logit[j] - m);
        denom += p;
        for (int c = 0; c < d; ++c) o[c] += p * bf16_to_f32(v[(static_cast<size_t>(h) * T + j) * d + c]);
      }
      for (int c = 0; c < d; ++c) out[(static_cast<size_t>(h) * T + i) * d + c] = o[c] / denom;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Sec. 3.2, token importance.  In the paper's order:
//   pooled query   : special rows copied, patch rows averaged in consecutive groups of g
//                    (reading: a short last group is averaged over its real size)
//   head average   : Qbar = (1/H) sum_h pooled[h]                        [N_pooled][d]
//   key summary    : Kbar_j = (1/H) sum_h K[h][j]   over the prunable middle   [P][d]
//   score matrix   : S_matrix = Qbar Kbar^T                               [N_pooled][P]
//   importance     : S_j = (1/N_pooled) sum_i S_matrix[i][j]              [P]
//   q [H][n][d] bf16 (n_s special rows first);  k_mid [H][P][d] bf16;  scores [P].
// Returns N_pooled.
int xsv_ref_score(const uint16_t* q, const uint16_t* k_mid, int H, int n, int n_s, int P, int d,
                  int g, float* scores) {
  const int n_patch = n - n_s;
  const int n_pooled = n_s + ceil_div(n_patch, g);
  std::vector<float> pooled(static_cast<size_t>(H) * n_pooled * d);
  for (int h = 0; h < H; ++h) {
    for (int i = 0; i < n_s; ++i)
      for (int c = 0; c < d; ++c)
        pooled[(static_cast<size_t>(h) * n_pooled + i) * d + c] =
            bf16_to_f32(q[(static_cast<size_t>(h) * n + i) * d + c]);
    for (int u = 0; u < n_pooled - n_s; ++u) {
      const int r0 = n_s + u * g, r1 = std::min(n, r0 + g);
      for (int c = 0; c < d; ++c) {
        float acc = 0.0f;
        for (int r = r0; r < r1; ++r) acc += bf16_to_f32(q[(static_cast<size_t>(h) * n + r) * d + c]);
        pooled[(static_cast<size_t>(h) * n_pooled + n_s + u) * d + c] = acc / static_cast<float>(r1 - r0);
      }
    }
  }
  std::vector<float> qbar(static_cast<size_t>(n_pooled) * d);
  for (int i = 0; i < n_pooled; ++i)
    for (int c = 0; c < d; ++c) {
      float acc = 0.0f;
      for (int h = 0; h < H; ++h) acc += pooled[(static_cast<size_t>(h) * n_pooled + i) * d + c];
      qbar[static_cast<size_t>(i) * d + c] = acc / static_cast<float>(H);
    }
  std::vector<float> kbar(static_cast<size_t>(P) * d);
  for (int j = 0; j < P; ++j)
    for (int c = 0; c < d; ++c) {
      float acc = 0.0f;
      for (int h = 0; h < H; ++h) acc += bf16_to_f32(k_mid[(static_cast<size_t>(h) * P + j) * d + c]);
      kbar[static_cast<size_t>(j) * d + c] = acc / static_cast<float>(H);
    }
#pragma omp parallel for schedule(static)
  for (int j = 0; j < P; ++j) {
    float total = 0.0f;
    for (int i = 0; i < n_pooled; ++i) {
      float dot = 0.0f;
      for (int c = 0; c < d; ++c) dot += qbar[static_cast<size_t>(i) * d + c] * kbar[static_cast<size_t>(j) * d + c];
      total += dot;
    }
    scores[j] = total / static_cast<float>(n_pooled);
  }
  return n_pooled;
}

// Sec. 3.2, retained index set: first frame, the k highest-scoring middle tokens, current frame.
// Readings: equal scores → the smaller index wins; the result is listed in ascending position.
//   scores [P] are for positions T_first .. T_first+P-1;  keep has T_first + k + T_cur entries.
void xsv_ref_select(const float* scores, int P, int k, int T_first, int T_cur, int32_t* keep) {
  std::vector<int32_t> order(P);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return scores[a] > scores[b]; });
  std::vector<int32_t> chosen(order.begin(), order.begin() + k);
  std::sort(chosen.begin(), chosen.end());
  int32_t* w = keep;
  for (int i = 0; i < T_first; ++i) *w++ = i;
  for (int32_t j : chosen) *w++ = T_first + j;
  for (int i = 0; i < T_cur; ++i) *w++ = T_first + P + i;
}

// ------------------------------------------------------------------------------------------------
// The streaming state: one cache per layer, stepped frame by frame.
struct xsv_ref_config {
  int32_t n_layers, n_heads, head_dim;
  int32_t tokens_per_frame, n_special;
  int32_t budget;      // L_max per head per layer; 0 = unbounded
  int32_t kv_bits;     // 2, 4, or 16 (= bf16 cache, no quantization)
  int32_t group_size;  // G
  int32_t pool_size;   // g
  float softmax_scale;  // 0 → 1/sqrt(head_dim)
  // 0: the paper's score (Sec. 3.2: queries and keys averaged over the heads, ONE retained index set
  //    per layer, shared by all heads).
  // 1: a variant, not the paper's: the head averages are left out, every head scores its own keys
  //    with its own pooled queries and keeps its own top-k.  All heads still keep the same NUMBER of
  //    tokens, so the cache length stays one number per layer.
  int32_t score_mode;
  // 0: the whole retained cache is quantized anew every step (the reading of Sec. 3.3 used throughout: quantization is
  //    applied to the final cache, history through its dequantized view).
  // 1: a variant, "quantize once" for the values: a value row is quantized when its frame is appended, and a row that
  //    is retained keeps those codes, its scale and its zero point for as long as it stays in the cache (a value row's
  //    groups are its own channels, so nothing about them depends on which other tokens are retained).  Keys are
  //    quantized anew as in mode 0: their groups are runs of consecutive RETAINED tokens and change with every pruning.
  int32_t value_mode;
};

// "sets" below = index sets per layer: 1 (score_mode 0) or H (score_mode 1, set s belongs to head s).
struct RefLayer {
  int T = 0, T_first = 0, frames = 0;
  std::vector<uint8_t> k_codes, v_codes;        // [H][T][d]
  std::vector<float> k_scale, k_zero;           // [H][ceil(T/G)][d]
  std::vector<float> v_scale, v_zero;           // [H][T][d/G]
  std::vector<uint16_t> k_bf16, v_bf16;         // [H][T][d] when kv_bits == 16
  std::vector<int32_t> token_frame, token_index;  // [sets][T]
  std::vector<float> last_scores;               // [sets][P] of the last step that scored
  std::vector<int32_t> last_keep;               // [sets][T'] positions in [cache ; frame] kept by the last step
};

struct xsv_ref_state {
  xsv_ref_config cfg;
  std::vector<RefLayer> layers;
};

xsv_ref_state* xsv_ref_create(const xsv_ref_config* cfg) {
  if (!cfg || cfg->n_layers <= 0 || cfg->n_heads <= 0 || cfg->head_dim <= 0) return nullptr;
  if (cfg->kv_bits != 2 && cfg->kv_bits != 4 && cfg->kv_bits != 16) return nullptr;
  if (cfg->kv_bits != 16 && (cfg->group_size <= 0 || cfg->head_dim % cfg->group_size != 0)) return nullptr;
  if (cfg->score_mode != 0 && cfg->score_mode != 1) return nullptr;
  if (cfg->value_mode != 0 && cfg->value_mode != 1) return nullptr;
  auto* st = new xsv_ref_state;
  st->cfg = *cfg;
  if (st->cfg.softmax_scale == 0.0f) st->cfg.softmax_scale = 1.0f / std::sqrt(static_cast<float>(cfg->head_dim));
  st->layers.resize(cfg->n_layers);
  return st;
}

void xsv_ref_destroy(xsv_ref_state* st) { delete st; }

int xsv_ref_num_sets(const xsv_ref_state* st) { return st->cfg.score_mode == 1 ? st->cfg.n_heads : 1; }
int xsv_ref_cache_len(const xsv_ref_state* st, int layer) { return st->layers[layer].T; }
// entries PER SET of the last step's scores / keep list
int xsv_ref_last_scores_len(const xsv_ref_state* st, int layer) {
  return static_cast<int>(st->layers[layer].last_scores.size()) / xsv_ref_num_sets(st);
}
int xsv_ref_last_keep_len(const xsv_ref_state* st, int layer) {
  return static_cast<int>(st->layers[layer].last_keep.size()) / xsv_ref_num_sets(st);
}

// The bf16 view of a layer's cache: (code - z) * s rounded to bf16, or the stored rows (bits 16).
void xsv_ref_cache_view(const xsv_ref_state* st, int layer, uint16_t* k_out, uint16_t* v_out) {
  const xsv_ref_config& c = st->cfg;
  const RefLayer& L = st->layers[layer];
  const size_t count = static_cast<size_t>(c.n_heads) * L.T * c.head_dim;
  if (L.T == 0) return;
  if (c.kv_bits == 16) {
    copy_bytes(k_out, L.k_bf16.data(), count * 2);
    copy_bytes(v_out, L.v_bf16.data(), count * 2);
  } else {
    xsv_ref_dequantize_k(L.k_codes.data(), L.k_scale.data(), L.k_zero.data(), c.n_heads, L.T, c.head_dim,
                         c.group_size, k_out);
    xsv_ref_dequantize_v(L.v_codes.data(), L.v_scale.data(), L.v_zero.data(), c.n_heads, L.T, c.head_dim,
                         c.group_size, v_out);
  }
}

// One streaming step of one layer for frame t (Sec. 3.1-3.3, in the order of the method's
// overview figure): attend → append → (score → select, once the length exceeds the budget) →
// gather → quantize the whole retained cache.
//   q, k_new, v_new [H][n][d] bf16
//   rows/n_rows/out: attention is evaluated for these query rows only (rows NULL → all;
//                    out NULL → attention skipped; the cache never depends on the output)
//   forced_keep: when non-NULL ([sets][n_forced], each list ascending positions in [cache ; frame])
//                it replaces the selection — used to adopt a documented near-tie decision.
// Returns the new cache length, or a negative value on a bad argument.
int xsv_ref_step(xsv_ref_state* st, int layer, const uint16_t* q, const uint16_t* k_new,
                 const uint16_t* v_new, const int32_t* rows, int n_rows, float* out,
                 const int32_t* forced_keep, int n_forced) {
  if (!st || layer < 0 || layer >= st->cfg.n_layers) return -1;
  const xsv_ref_config& c = st->cfg;
  RefLayer& L = st->layers[layer];
  const int H = c.n_heads, d = c.head_dim, n = c.tokens_per_frame;
  const int Tc = L.T, T = Tc + n;
  const int sets = xsv_ref_num_sets(st);

  // [cache view ; current frame], per head.
  std::vector<uint16_t> k_all(static_cast<size_t>(H) * T * d), v_all(static_cast<size_t>(H) * T * d);
  {
    std::vector<uint16_t> k_view(static_cast<size_t>(H) * Tc * d), v_view(static_cast<size_t>(H) * Tc * d);
    xsv_ref_cache_view(st, layer, k_view.data(), v_view.data());
    for (int h = 0; h < H; ++h) {
      copy_bytes(k_all.data() + static_cast<size_t>(h) * T * d, k_view.data() + static_cast<size_t>(h) * Tc * d,
                  static_cast<size_t>(Tc) * d * 2);
      copy_bytes(v_all.data() + static_cast<size_t>(h) * T * d, v_view.data() + static_cast<size_t>(h) * Tc * d,
                  static_cast<size_t>(Tc) * d * 2);
      copy_bytes(k_all.data() + (static_cast<size_t>(h) * T + Tc) * d, &k_new[static_cast<size_t>(h) * n * d],
                  static_cast<size_t>(n) * d * 2);
      copy_bytes(v_all.data() + (static_cast<size_t>(h) * T + Tc) * d, &v_new[static_cast<size_t>(h) * n * d],
                  static_cast<size_t>(n) * d * 2);
    }
  }

  // Sec. 3.1: attention of frame t over everything cached plus itself.
  if (out != nullptr) xsv_ref_attend(q, k_all.data(), v_all.data(), H, n, T, d, c.softmax_scale, rows, n_rows, out);

  // Sec. 3.1: append.
  const int frame_id = L.frames;
  if (L.frames == 0) L.T_first = n;
  const int T_first = L.T_first, T_cur = n;

  // Sec. 3.2: prune once T exceeds the budget; first and current frames are always kept.
  // One index set per layer (score_mode 0) or one per head (score_mode 1).
  std::vector<std::vector<int32_t>> keep(sets);
  L.last_scores.clear();
  if (forced_keep != nullptr) {
    for (int s = 0; s < sets; ++s)
      keep[s].assign(forced_keep + static_cast<size_t>(s) * n_forced, forced_keep + static_cast<size_t>(s + 1) * n_forced);
  } else if (c.budget == 0 || T <= c.budget || L.frames == 0) {
    for (int s = 0; s < sets; ++s) {
      keep[s].resize(T);
      std::iota(keep[s].begin(), keep[s].end(), 0);
    }
  } else {
    const int P = T - T_first - T_cur;
    int k = std::max(0, c.budget - T_first - T_cur);
    k = std::min(k, P);
    const bool scored = k > 0 && k < P;
    for (int s = 0; s < sets; ++s) {
      std::vector<float> scores(P);
      if (scored) {
        if (c.score_mode == 0) {
          std::vector<uint16_t> k_mid(static_cast<size_t>(H) * P * d);
          for (int h = 0; h < H; ++h)
            copy_bytes(k_mid.data() + static_cast<size_t>(h) * P * d, k_all.data() + (static_cast<size_t>(h) * T + T_first) * d,
                        static_cast<size_t>(P) * d * 2);
          xsv_ref_score(q, k_mid.data(), H, n, c.n_special, P, d, c.pool_size, scores.data());
        } else {
          // head s alone: the same score with "all heads" = this one head
          xsv_ref_score(q + static_cast<size_t>(s) * n * d, k_all.data() + (static_cast<size_t>(s) * T + T_first) * d, 1, n,
                        c.n_special, P, d, c.pool_size, scores.data());
        }
        L.last_scores.insert(L.last_scores.end(), scores.begin(), scores.end());
      }
      keep[s].resize(T_first + k + T_cur);
      xsv_ref_select(scores.data(), P, k, T_first, T_cur, keep[s].data());
    }
  }
  const int Tn = static_cast<int>(keep[0].size());
  L.last_keep.clear();
  for (int s = 0; s < sets; ++s) {
    if (static_cast<int>(keep[s].size()) != Tn) return -2;
    for (int i = 0; i < Tn; ++i)
      if (keep[s][i] < 0 || keep[s][i] >= T || (i > 0 && keep[s][i] <= keep[s][i - 1])) return -2;
    L.last_keep.insert(L.last_keep.end(), keep[s].begin(), keep[s].end());
  }

  // Gather the retained rows (same indices for keys and values) and their token ids.
  std::vector<uint16_t> k_kept(static_cast<size_t>(H) * Tn * d), v_kept(static_cast<size_t>(H) * Tn * d);
  for (int h = 0; h < H; ++h) {
    const std::vector<int32_t>& kp = keep[sets == 1 ? 0 : h];
    for (int i = 0; i < Tn; ++i) {
      copy_bytes(k_kept.data() + (static_cast<size_t>(h) * Tn + i) * d, k_all.data() + (static_cast<size_t>(h) * T + kp[i]) * d, d * 2);
      copy_bytes(v_kept.data() + (static_cast<size_t>(h) * Tn + i) * d, v_all.data() + (static_cast<size_t>(h) * T + kp[i]) * d, d * 2);
    }
  }
  std::vector<int32_t> tf(static_cast<size_t>(sets) * Tn), ti(static_cast<size_t>(sets) * Tn);
  for (int s = 0; s < sets; ++s)
    for (int i = 0; i < Tn; ++i) {
      const int src = keep[s][i];
      if (src < Tc) {
        tf[static_cast<size_t>(s) * Tn + i] = L.token_frame[static_cast<size_t>(s) * Tc + src];
        ti[static_cast<size_t>(s) * Tn + i] = L.token_index[static_cast<size_t>(s) * Tc + src];
      } else {
        tf[static_cast<size_t>(s) * Tn + i] = frame_id;
        ti[static_cast<size_t>(s) * Tn + i] = src - Tc;
      }
    }
  L.token_frame.swap(tf);
  L.token_index.swap(ti);

  // Sec. 3.3: quantize the final cache (pruned history + first + current frames), every step.
  if (c.kv_bits == 16) {
    L.k_bf16.swap(k_kept);
    L.v_bf16.swap(v_kept);
  } else {
    const int G = c.group_size;
    const size_t n_el = static_cast<size_t>(H) * Tn * d;
    // (value_mode 1: what the retained rows held before this step, to be put back below)
    std::vector<uint8_t> v_codes_old;
    std::vector<float> v_scale_old, v_zero_old;
    if (c.value_mode == 1) {
      v_codes_old = L.v_codes;
      v_scale_old = L.v_scale;
      v_zero_old = L.v_zero;
    }
    L.k_codes.assign(n_el, 0);
    L.v_codes.assign(n_el, 0);
    L.k_scale.assign(static_cast<size_t>(H) * ceil_div(Tn, G) * d, 0.0f);
    L.k_zero.assign(L.k_scale.size(), 0.0f);
    L.v_scale.assign(static_cast<size_t>(H) * Tn * (d / G), 0.0f);
    L.v_zero.assign(L.v_scale.size(), 0.0f);
    xsv_ref_quantize_k(k_kept.data(), H, Tn, d, c.kv_bits, G, L.k_codes.data(), L.k_scale.data(), L.k_zero.data());
    xsv_ref_quantize_v(v_kept.data(), H, Tn, d, c.kv_bits, G, L.v_codes.data(), L.v_scale.data(), L.v_zero.data());
    if (c.value_mode == 1) {
      // quantize once: a row that came from the cache keeps the codes and parameters it had there
      const int vg = d / G;
      for (int h = 0; h < H; ++h) {
        const std::vector<int32_t>& kp = keep[sets == 1 ? 0 : h];
        for (int i = 0; i < Tn; ++i) {
          const int src = kp[i];
          if (src >= Tc) continue;  // a row of the current frame: quantized just now, for good
          for (int ch = 0; ch < d; ++ch)
            L.v_codes[(static_cast<size_t>(h) * Tn + i) * d + ch] = v_codes_old[(static_cast<size_t>(h) * Tc + src) * d + ch];
          for (int g = 0; g < vg; ++g) {
            L.v_scale[(static_cast<size_t>(h) * Tn + i) * vg + g] = v_scale_old[(static_cast<size_t>(h) * Tc + src) * vg + g];
            L.v_zero[(static_cast<size_t>(h) * Tn + i) * vg + g] = v_zero_old[(static_cast<size_t>(h) * Tc + src) * vg + g];
          }
        }
      }
    }
  }
  L.T = Tn;
  L.frames += 1;
  return Tn;
}

// Copies of the layer's state, any pointer may be NULL.  Shapes as documented on RefLayer.
void xsv_ref_export(const xsv_ref_state* st, int layer, uint8_t* k_codes, float* k_scale, float* k_zero,
                    uint8_t* v_codes, float* v_scale, float* v_zero, uint16_t* k_bf16, uint16_t* v_bf16,
                    int32_t* token_frame, int32_t* token_index, float* last_scores, int32_t* last_keep) {
  const RefLayer& L = st->layers[layer];
  auto cp = [](auto* dst, const auto& src) {
    if (dst && !src.empty()) copy_bytes(dst, src.data(), src.size() * sizeof(src[0]));
  };
  cp(k_codes, L.k_codes);
  cp(k_scale, L.k_scale);
  cp(k_zero, L.k_zero);
  cp(v_codes, L.v_codes);
  cp(v_scale, L.v_scale);
  cp(v_zero, L.v_zero);
  cp(k_bf16, L.k_bf16);
  cp(v_bf16, L.v_bf16);
  cp(token_frame, L.token_frame);
  cp(token_index, L.token_index);
  cp(last_scores, L.last_scores);
  cp(last_keep, L.last_keep);
}

// Threads the OpenMP loops above run on (reported beside timings).
int xsv_ref_num_threads() {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

}  // extern "C"
