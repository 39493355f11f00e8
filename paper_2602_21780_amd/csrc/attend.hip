// Fused dequantize + flash-style attention of one frame's queries over [packed cache ; frame]
// (paper Sec. 3.1 temporal attention, Sec. 3.3 dequantization at attention time) for gfx950.
//
// Work decomposition
//   workgroup = NW waves; each wave owns 32 query rows of one head and keeps, per lane, the
//   transposed tiles  S^T = K Q^T  (64 tokens x 32 queries)  and  O^T = V^T P^T  (64 channels x 32
//   queries) in MFMA 32x32x16 bf16 accumulators.  In this orientation one lane holds 32 logits of
//   ONE query, so the online-softmax row reductions are in-lane plus one exchange with lane^32, and
//   the exponentiated tile is already laid out as the B operand of the PV product — provided the
//   key rows of the first product are read in a permuted order (tau below), which costs nothing.
//   The workgroup walks the key axis in tiles of 64 tokens.  All waves cooperatively dequantize a
//   tile ONCE into LDS as bf16 (K row-major [token][channel], V transposed [channel][token], the
//   layout the packed cache already has), so the unpack/convert cost is shared by NW*32 queries.
//   LDS is double buffered; the next tile's packed codes and group parameters are fetched into
//   registers before the current tile's MFMAs are issued.
//   blockIdx is remapped so that all query blocks of one (layer, head, key range) land on the same
//   XCD and share its L2.  With n_splits > 1 each key range writes unnormalized partials that
//   combine_kernel merges.
#include "xsv_internal.h"

namespace xsv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kLdsStride = 72;  // bf16 elements per LDS row: 64 + 8 pad (144 B, keeps 16 B alignment)
constexpr float kNegBig = -1.0e30f;

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  __bf16 x = (__bf16)a, y = (__bf16)b;  // round to nearest even (v_cvt_pk_bf16_f32)
  return (uint32_t)__builtin_bit_cast(unsigned short, x) | ((uint32_t)__builtin_bit_cast(unsigned short, y) << 16);
}

// Row of the K tile that MFMA row i of S^T reads, so that accumulator register r of the lane
// half hh holds token 16*(r/8) + 8*hh + r%8 — the order in which the PV product consumes tokens.
__device__ __forceinline__ int tau(int i) {
  const int a = i >> 3;
  return 16 * (a >> 1) + 8 * ((i >> 2) & 1) + 4 * (a & 1) + (i & 3);
}

// ---- staging of one key tile -------------------------------------------------------------------
// Raw (still packed) data of the items one thread stages, fetched ahead of use.
template <int BITS, int G, int NT>
struct Staged {
  static constexpr int kDw = (BITS == 16) ? 4 : 1;                    // dwords per item
  static constexpr int kPer = (BITS == 16) ? 8 : 32 / BITS;           // elements per item
  static constexpr int kItems = kTile * kD / kPer;                    // items per tile (K, same for V)
  static constexpr int kRowItems = kD / kPer;                         // items per K row / V block row
  static constexpr int kIter = (kItems + NT - 1) / NT;
  uint32_t k[kIter][4];
  uint32_t v[kIter][4];
  float ks[kIter][kPer > 8 ? 16 : 8], kz[kIter][kPer > 8 ? 16 : 8];
  float vs[kIter][kPer > 8 ? 16 : 8], vz[kIter][kPer > 8 ? 16 : 8];
};

// A tile either comes from the packed cache (CACHE = true) or from the frame's own bf16 K/V.
template <int BITS, int G, int NT>
__device__ __forceinline__ void fetch_cache_tile(Staged<BITS, G, NT>& st, const CachePool& pool,
                                                 const LayerCache& lc, int h, int tile, int tid) {
  using S = Staged<BITS, G, NT>;
  constexpr int kRowDw = kD * BITS / 32;  // dwords per K row == dwords per V block row
  const uint32_t* kc = reinterpret_cast<const uint32_t*>(lc.kc) + ((size_t)h * pool.Tcap + (size_t)tile * kTile) * kRowDw;
  const uint32_t* vc = reinterpret_cast<const uint32_t*>(lc.vc) + ((size_t)h * pool.Tcap + (size_t)tile * kTile) * kRowDw;
#pragma unroll
  for (int it = 0; it < S::kIter; ++it) {
    const int i = tid + it * NT;
    if (S::kItems % NT != 0 && i >= S::kItems) break;
    if constexpr (BITS == 16) {
      const uint4 a = reinterpret_cast<const uint4*>(kc)[i];
      const uint4 b = reinterpret_cast<const uint4*>(vc)[i];
      st.k[it][0] = a.x; st.k[it][1] = a.y; st.k[it][2] = a.z; st.k[it][3] = a.w;
      st.v[it][0] = b.x; st.v[it][1] = b.y; st.v[it][2] = b.z; st.v[it][3] = b.w;
    } else {
      st.k[it][0] = kc[i];
      st.v[it][0] = vc[i];
      // K item = (token r, channel run o*kPer..): parameters per channel, group of the token
      const int r = i / S::kRowItems, o = i % S::kRowItems;
      const int grp = (G >= kTile) ? tile / (G / kTile) : tile * (kTile / G) + r / G;
      const float* ks = lc.ks + ((size_t)h * (pool.Tcap / G) + grp) * kD + o * S::kPer;
      const float* kz = lc.kz + ((size_t)h * (pool.Tcap / G) + grp) * kD + o * S::kPer;
      // V item = (channel c, token run o*kPer..): parameters per token, group of the channel
      const int cg = (G >= kD) ? 0 : r / G;  // r is the channel here
      const float* vs = lc.vs + ((size_t)h * pool.Tcap + (size_t)tile * kTile + o * S::kPer) * (kD / G) + cg;
      const float* vz = lc.vz + ((size_t)h * pool.Tcap + (size_t)tile * kTile + o * S::kPer) * (kD / G) + cg;
#pragma unroll
      for (int e = 0; e < S::kPer; ++e) {
        st.ks[it][e] = ks[e];
        st.kz[it][e] = kz[e];
        st.vs[it][e] = vs[e * (kD / G)];
        st.vz[it][e] = vz[e * (kD / G)];
      }
    }
  }
}

template <int BITS, int G, int NT>
__device__ __forceinline__ void store_cache_tile(const Staged<BITS, G, NT>& st, uint16_t* lk, uint16_t* lv, int tid) {
  using S = Staged<BITS, G, NT>;
#pragma unroll
  for (int it = 0; it < S::kIter; ++it) {
    const int i = tid + it * NT;
    if (S::kItems % NT != 0 && i >= S::kItems) break;
    const int r = i / S::kRowItems, o = i % S::kRowItems;  // K: token r, run o;  V: channel r, token run o
    if constexpr (BITS == 16) {
      *reinterpret_cast<uint4*>(lk + r * kLdsStride + o * 8) = make_uint4(st.k[it][0], st.k[it][1], st.k[it][2], st.k[it][3]);
      *reinterpret_cast<uint4*>(lv + r * kLdsStride + o * 8) = make_uint4(st.v[it][0], st.v[it][1], st.v[it][2], st.v[it][3]);
    } else {
      constexpr uint32_t mask = (1u << BITS) - 1u;
      uint32_t pk[S::kPer / 2], pv[S::kPer / 2];
#pragma unroll
      for (int e = 0; e < S::kPer; e += 2) {
        // the cache's view of a stored element: (code - zero) * scale, then bf16
        const float k0 = ((float)((st.k[it][0] >> (BITS * e)) & mask) - st.kz[it][e]) * st.ks[it][e];
        const float k1 = ((float)((st.k[it][0] >> (BITS * (e + 1))) & mask) - st.kz[it][e + 1]) * st.ks[it][e + 1];
        const float v0 = ((float)((st.v[it][0] >> (BITS * e)) & mask) - st.vz[it][e]) * st.vs[it][e];
        const float v1 = ((float)((st.v[it][0] >> (BITS * (e + 1))) & mask) - st.vz[it][e + 1]) * st.vs[it][e + 1];
        pk[e / 2] = pack_bf16(k0, k1);
        pv[e / 2] = pack_bf16(v0, v1);
      }
#pragma unroll
      for (int w = 0; w < S::kPer / 8; ++w) {
        *reinterpret_cast<uint4*>(lk + r * kLdsStride + o * S::kPer + w * 8) = make_uint4(pk[4 * w], pk[4 * w + 1], pk[4 * w + 2], pk[4 * w + 3]);
        *reinterpret_cast<uint4*>(lv + r * kLdsStride + o * S::kPer + w * 8) = make_uint4(pv[4 * w], pv[4 * w + 1], pv[4 * w + 2], pv[4 * w + 3]);
      }
    }
  }
}

// Frame tiles: 512 items of 8 bf16, item = (token r, channel run o).
template <int NT>
struct StagedFrame {
  static constexpr int kIter = (512 + NT - 1) / NT;
  uint4 k[kIter], v[kIter];
};

template <int NT>
__device__ __forceinline__ void fetch_frame_tile(StagedFrame<NT>& st, const uint16_t* kh, const uint16_t* vh,
                                                 int64_t k_st, int64_t v_st, int tile, int n, int tid) {
#pragma unroll
  for (int it = 0; it < StagedFrame<NT>::kIter; ++it) {
    const int i = tid + it * NT;
    const int r = i >> 3, o = i & 7;
    const int row = tile * kTile + r;
    if (row < n) {
      st.k[it] = *reinterpret_cast<const uint4*>(kh + (size_t)row * k_st + o * 8);
      st.v[it] = *reinterpret_cast<const uint4*>(vh + (size_t)row * v_st + o * 8);
    } else {  // rows past the frame: zeros (their logits are masked, their values must be finite)
      st.k[it] = make_uint4(0, 0, 0, 0);
      st.v[it] = make_uint4(0, 0, 0, 0);
    }
  }
}

template <int NT>
__device__ __forceinline__ void store_frame_tile(const StagedFrame<NT>& st, uint16_t* lk, uint16_t* lv, int tid) {
#pragma unroll
  for (int it = 0; it < StagedFrame<NT>::kIter; ++it) {
    const int i = tid + it * NT;
    const int r = i >> 3, o = i & 7;
    *reinterpret_cast<uint4*>(lk + r * kLdsStride + o * 8) = st.k[it];
    // V goes in transposed: element (token r, channel 8o+e) → row 8o+e, column r
    const uint32_t w[4] = {st.v[it].x, st.v[it].y, st.v[it].z, st.v[it].w};
#pragma unroll
    for (int e = 0; e < 8; ++e)
      lv[(o * 8 + e) * kLdsStride + r] = (uint16_t)((e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xffffu));
  }
}

// ---- the kernel ----------------------------------------------------------------------------------
template <int BITS, int G, int NW>
__global__ __launch_bounds__(NW * 64) void attend_kernel(const AttendArgs a) {
  constexpr int NT = NW * 64;
  __shared__ __attribute__((aligned(16))) uint16_t lds_k[2][kTile * kLdsStride];
  __shared__ __attribute__((aligned(16))) uint16_t lds_v[2][kD * kLdsStride];

  const int H = a.pool.H, n = a.n, Tc = a.Tc, S = a.n_splits;
  const int nqb = (n + 32 * NW - 1) / (32 * NW);
  const int n_groups = a.b.n_layers * H * S;
  // XCD-aware decode: ids with equal (id % 8) run on the same XCD; give them the same keys.
  const int id = blockIdx.x;
  const int chunk = id / (8 * nqb), within = id % (8 * nqb);
  const int grp = chunk * 8 + (within & 7);
  const int qb = within >> 3;
  if (grp >= n_groups) return;
  const int split = grp % S;
  const int h = (grp / S) % H;
  const int lb = grp / (S * H);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int j = lane & 31, hh = lane >> 5;

  const LayerCache lc = layer_cache(a.pool, a.b.src_buf(lb), a.b.layer0 + lb);
  const uint16_t* qh = a.b.q[lb] + (size_t)h * a.b.q_sh;
  const uint16_t* kh = a.b.k[lb] + (size_t)h * a.b.k_sh;
  const uint16_t* vh = a.b.v[lb] + (size_t)h * a.b.v_sh;

  // tiles: cache blocks first, then the frame's own tokens (each range padded to 64 on its own)
  const int n_ct = (Tc + kTile - 1) / kTile, n_ft = (n + kTile - 1) / kTile;
  const int n_tiles = n_ct + n_ft;
  const int t_begin = (int)((long long)n_tiles * split / S), t_end = (int)((long long)n_tiles * (split + 1) / S);

  // query fragments (B operand): lane holds channels 16*ks + 8*hh .. +8 of query row j, as given
  // (the softmax scale is applied to the fp32 logits, so no extra bf16 rounding enters)
  const int q_row = qb * 32 * NW + wave * 32 + j;
  const bool q_valid = q_row < n;
  bf16x8 qf[4];
  {
    const uint16_t* qp = qh + (size_t)(q_valid ? q_row : n - 1) * a.b.q_st;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      qf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qp + 16 * ks + 8 * hh));
  }
  const float c2 = a.qscale;  // softmax scale * log2(e): p = 2^(c2 * (logit - max))

  f32x16 o0, o1;
#pragma unroll
  for (int r = 0; r < 16; ++r) { o0[r] = 0.f; o1[r] = 0.f; }
  float m = kNegBig, l = 0.f;  // running max of the raw logits and this lane's share of the row sum

  Staged<BITS, G, NT> sc;
  StagedFrame<NT> sf;
  auto fetch = [&](int t) {
    if (t < n_ct) fetch_cache_tile<BITS, G, NT>(sc, a.pool, lc, h, t, tid);
    else fetch_frame_tile<NT>(sf, kh, vh, a.b.k_st, a.b.v_st, t - n_ct, n, tid);
  };
  auto store = [&](int t, int buf) {
    if (t < n_ct) store_cache_tile<BITS, G, NT>(sc, lds_k[buf], lds_v[buf], tid);
    else store_frame_tile<NT>(sf, lds_k[buf], lds_v[buf], tid);
  };

  if (t_begin < t_end) {
    fetch(t_begin);
    store(t_begin, 0);
  }
  const int krow = tau(j);
  int cur = 0;
  for (int t = t_begin; t < t_end; ++t) {
    __syncthreads();  // tile t is in lds[cur]; everybody is done reading lds[cur^1]
    if (t + 1 < t_end) fetch(t + 1);

    const uint16_t* lk = lds_k[cur];
    const uint16_t* lv = lds_v[cur];
    f32x16 s0, s1;
#pragma unroll
    for (int r = 0; r < 16; ++r) { s0[r] = 0.f; s1[r] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(lk + krow * kLdsStride + 16 * ks + 8 * hh);
      const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(lk + (32 + krow) * kLdsStride + 16 * ks + 8 * hh);
      s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qf[ks], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qf[ks], s1, 0, 0, 0);
    }
    // tokens past the end of the cache / of the frame in a ragged tile
    const int valid = (t < n_ct) ? min(kTile, Tc - t * kTile) : min(kTile, n - (t - n_ct) * kTile);
    if (valid < kTile) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int tok = 16 * (r >> 3) + 8 * hh + (r & 7);
        if (tok >= valid) s0[r] = -INFINITY;
        if (tok + 32 >= valid) s1[r] = -INFINITY;
      }
    }
    // online softmax; the exponent is evaluated in base 2
    float mx = s0[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s0[r]);
#pragma unroll
    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s1[r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m, mx);
    if (__any(m_new > m)) {
      const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c2);
      l *= alpha;
#pragma unroll
      for (int r = 0; r < 16; ++r) { o0[r] *= alpha; o1[r] *= alpha; }
      m = m_new;
    }
    float psum = 0.f;
    const float mc = -m * c2;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      s0[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s0[r], c2, mc));
      s1[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s1[r], c2, mc));
      psum += s0[r] + s1[r];
    }
    l += psum;
    // O^T += V^T P^T: 4 contraction steps of 16 tokens; P comes straight from the accumulators
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      uint32_t pw[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int r = 8 * (ks & 1) + 2 * e;
        pw[e] = (ks < 2) ? pack_bf16(s0[r], s0[r + 1]) : pack_bf16(s1[r], s1[r + 1]);
      }
      const bf16x8 pb = __builtin_bit_cast(bf16x8, make_uint4(pw[0], pw[1], pw[2], pw[3]));
      const bf16x8 v0 = *reinterpret_cast<const bf16x8*>(lv + j * kLdsStride + 16 * ks + 8 * hh);
      const bf16x8 v1 = *reinterpret_cast<const bf16x8*>(lv + (32 + j) * kLdsStride + 16 * ks + 8 * hh);
      o0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v0, pb, o0, 0, 0, 0);
      o1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v1, pb, o1, 0, 0, 0);
    }

    if (t + 1 < t_end) store(t + 1, cur ^ 1);
    cur ^= 1;
  }

  l += __shfl_xor(l, 32);  // the two lane halves saw disjoint tokens of the same query
  if (!q_valid) return;
  // accumulator register r of o0 (o1) is channel 8*(r/4) + 4*hh + r%4 (+32) of query row j
  if (S == 1) {
    const float inv = 1.0f / l;
    uint16_t* op = a.b.out[lb] + ((size_t)h * n + q_row) * kD;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int c = 8 * q4 + 4 * hh;
      *reinterpret_cast<uint2*>(op + c) = make_uint2(pack_bf16(o0[4 * q4] * inv, o0[4 * q4 + 1] * inv),
                                                     pack_bf16(o0[4 * q4 + 2] * inv, o0[4 * q4 + 3] * inv));
      *reinterpret_cast<uint2*>(op + 32 + c) = make_uint2(pack_bf16(o1[4 * q4] * inv, o1[4 * q4 + 1] * inv),
                                                          pack_bf16(o1[4 * q4 + 2] * inv, o1[4 * q4 + 3] * inv));
    }
  } else {
    const size_t row = (((size_t)split * a.b.n_layers + lb) * H + h) * n + q_row;
    float* op = a.ws.attn_o + row * kD;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int c = 8 * q4 + 4 * hh;
      *reinterpret_cast<float4*>(op + c) = make_float4(o0[4 * q4], o0[4 * q4 + 1], o0[4 * q4 + 2], o0[4 * q4 + 3]);
      *reinterpret_cast<float4*>(op + 32 + c) = make_float4(o1[4 * q4], o1[4 * q4 + 1], o1[4 * q4 + 2], o1[4 * q4 + 3]);
    }
    if (hh == 0) *reinterpret_cast<float2*>(a.ws.attn_ml + row * 2) = make_float2(m * c2, l);
  }
}

// Merge of the key-range partials: out = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s.
__global__ __launch_bounds__(256) void combine_kernel(const AttendArgs a) {
  const int H = a.pool.H, n = a.n, S = a.n_splits;
  const size_t rows = (size_t)a.b.n_layers * H * n;
  const size_t gid = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t row = gid >> 4;
  const int c = (int)(gid & 15) * 4;
  if (row >= rows) return;
  float M = kNegBig;
  for (int s = 0; s < S; ++s) M = fmaxf(M, a.ws.attn_ml[(s * rows + row) * 2]);
  float L = 0.f, acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < S; ++s) {
    const float2 ml = *reinterpret_cast<const float2*>(a.ws.attn_ml + (s * rows + row) * 2);
    const float w = __builtin_amdgcn_exp2f(ml.x - M);
    const float4 o = *reinterpret_cast<const float4*>(a.ws.attn_o + (s * rows + row) * kD + c);
    L += w * ml.y;
    acc[0] += w * o.x; acc[1] += w * o.y; acc[2] += w * o.z; acc[3] += w * o.w;
  }
  const float inv = 1.0f / L;
  const int lb = (int)(row / ((size_t)H * n));
  const size_t in_layer = row - (size_t)lb * H * n;
  *reinterpret_cast<uint2*>(a.b.out[lb] + in_layer * kD + c) =
      make_uint2(pack_bf16(acc[0] * inv, acc[1] * inv), pack_bf16(acc[2] * inv, acc[3] * inv));
}

template <int BITS, int G>
static hipError_t launch_attend_t(const AttendArgs& a, hipStream_t stream) {
  constexpr int NW = 4;
  const int nqb = (a.n + 32 * NW - 1) / (32 * NW);
  const int n_groups = a.b.n_layers * a.pool.H * a.n_splits;
  const int grid = ((n_groups + 7) / 8) * 8 * nqb;
  hipLaunchKernelGGL((attend_kernel<BITS, G, NW>), dim3(grid), dim3(NW * 64), 0, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (a.n_splits > 1) {
    const size_t threads = (size_t)a.b.n_layers * a.pool.H * a.n * 16;
    hipLaunchKernelGGL(combine_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream, a);
    e = hipGetLastError();
  }
  return e;
}

hipError_t launch_attend(const AttendArgs& a, hipStream_t stream) {
  const int bits = a.pool.bits, G = a.pool.G;
  if (bits == 16) return launch_attend_t<16, 64>(a, stream);
  if (bits == 4 && G == 64) return launch_attend_t<4, 64>(a, stream);
  if (bits == 4 && G == 32) return launch_attend_t<4, 32>(a, stream);
  if (bits == 2 && G == 64) return launch_attend_t<2, 64>(a, stream);
  if (bits == 2 && G == 32) return launch_attend_t<2, 32>(a, stream);
  return hipErrorInvalidValue;
}

}  // namespace xsv
