// Fused dequantize + flash-style attention of one frame's queries over [packed cache ; frame]
// (paper Sec. 3.1 temporal attention, Sec. 3.3 dequantization at attention time) for gfx950.
//
// Work decomposition
//   workgroup = NW waves; each wave owns QB blocks of 32 query rows of one head and keeps, per
//   lane, the transposed tiles  S^T = K Q^T  (32 tokens x 32 queries per block)  and
//   O^T = V^T P^T  (64 channels x 32 queries per block) in MFMA 32x32x16 bf16 accumulators.  In
//   this orientation one lane holds the logits of ONE query, so the online-softmax row reductions
//   are in-lane plus one exchange with lane^32, and the exponentiated tile is already laid out as
//   the B operand of the PV product — provided the key rows of the first product are read in a
//   permuted order (tau below), which costs nothing.  Every K / V fragment read from LDS feeds QB
//   MFMAs.
//   The workgroup walks the key axis in tiles of 64 tokens (two half-steps of 32).  All waves
//   cooperatively dequantize a tile ONCE into LDS as bf16 (K row-major [token][channel], V
//   transposed [channel][token], the layout the packed cache already has), so the unpack/convert
//   cost is shared by NW*QB*32 queries (half of the threads stage K, the other half V, with the
//   same code on mirrored layouts).  LDS is double buffered; the next tile's packed codes and
//   group parameters are fetched into registers before the current tile's MFMAs are issued.
//   Partition.  A unit is one (layer, head, block of NW*QB*32 query rows); its work is its key tiles.
//   Two forms, chosen by the host.  (a) Every unit is cut into the same number R of key ranges
//   (gridDim.x = units * R): the host passes where each range begins, placed so that the ranges cost
//   the same (a tile of the frame's own rows costs a little less than a cache tile, and the last
//   range may be made short on purpose so that its compute units are free early for the kernels
//   that run beside this one); the grid is permuted so that the query blocks of one (layer, head,
//   range), which read the same tiles, run on one XCD and share its L2.  (b) Otherwise all units'
//   tiles form one line of n_units * n_tiles items cut into gridDim.x equal pieces, so that any
//   number of workgroups gets the same amount of work; a piece may end one unit and begin the
//   next, and the workgroup handles them one after the other.  In both forms a unit covered by one
//   workgroup is normalized and written directly; otherwise each workgroup writes an unnormalized
//   partial that combine_kernel merges.
//   Softmax.  No row maximum on the common path: the reference of the exponent only moves when a
//   row sum leaves [0, 2^64] (which also catches the very first tile, whose reference is a
//   sentinel that sends every probability to +infinity); then, and only then, the maximum is
//   taken, the accumulators are rescaled and the block's probabilities are recomputed.
#include <cstddef>
#include <type_traits>

#include "xsv_internal.h"

namespace xsv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kLdsStride = 72;  // bf16 elements per LDS row: 64 + 8 pad (144 B, keeps 16 B alignment)
constexpr int kLdsTile = 64 * kLdsStride;  // elements of one K (or V) tile in LDS
constexpr float kNegBig = -1.0e30f;
// "no reference yet": with this in place of -reference every finite logit exponentiates to +infinity, which the
// row-sum check catches, and the first real reference then scales the (empty) sums by 2^-huge = 0
constexpr float kNoReference = 1.0e30f;
// row sums may grow to this before the reference of the exponent is moved: 2^64 leaves the fp32 accumulators
// (sums of probability x value over thousands of tokens) far from overflow
constexpr float kSumLimit = 0x1p64f;

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  const f32x2 v = {a, b};  // one v_cvt_pk_bf16_f32: round to nearest even, a in the low half
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
__device__ __forceinline__ uint32_t pack_f16(float a, float b) {
  const f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}

// Row of the K tile that MFMA row i of S^T reads, so that accumulator register r of the lane
// half hh holds token 16*(r/8) + 8*hh + r%8 — the order in which the PV product consumes tokens.
__device__ __forceinline__ int tau(int i) {
  const int a = i >> 3;
  return 16 * (a >> 1) + 8 * ((i >> 2) & 1) + 4 * (a & 1) + (i & 3);
}

// code e (0 .. 32/BITS-1) of a packed dword as float; the masks are shared between neighbours
template <int BITS>
__device__ __forceinline__ void unpack_codes(uint32_t w, float* out) {
  if constexpr (BITS == 4) {
    uint32_t t0 = w & 0x0f0f0f0fu, t1 = (w >> 4) & 0x0f0f0f0fu;
    // (opaque to the optimizer, which would otherwise fold the masks into one bit-field extract
    // PER code in front of each conversion instead of the byte-select conversions below)
    asm volatile("" : "+v"(t0), "+v"(t1));
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      out[2 * b] = (float)((t0 >> (8 * b)) & 0xffu);  // v_cvt_f32_ubyte<b>
      out[2 * b + 1] = (float)((t1 >> (8 * b)) & 0xffu);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint32_t t = (w >> (2 * i)) & 0x03030303u;
      asm volatile("" : "+v"(t));
#pragma unroll
      for (int b = 0; b < 4; ++b) out[4 * b + i] = (float)((t >> (8 * b)) & 0xffu);
    }
  }
}

// ---- staging of one key tile -------------------------------------------------------------------
// A tile is 64 tokens x 64 channels of K and of V.  It is cut into "items" of one dword of codes
// (8 or 16 elements; bf16 tiles: 16 bytes = 8 elements).  The first half of the workgroup's threads
// stages K, the second half V; both run the SAME code on different pointers, because the packed
// layouts mirror each other:  K item i = (token i / RI, channel run i % RI) with per-channel
// parameters,  V item i = (channel i / RI, token run i % RI) with per-token parameters, and the
// LDS tile of either is [row = i / RI][column run].  A thread stages items u, u + NH, .. (u = its
// index within its half, NH threads per half); NH is a multiple of RI, so all its items share the
// column run and (within a group) the parameters.
template <int BITS, int G, int NH>
struct Stage {
  static constexpr bool kQuant = BITS != 16;
  static constexpr int kPer = kQuant ? 32 / BITS : 8;  // elements per item
  static constexpr int kRI = kD / kPer;                 // items per row
  static constexpr int kItems = kTile * kRI;            // per tile and role
  static constexpr int kIter = kItems / NH;             // items per thread
  static constexpr int kRowStep = NH / kRI;             // rows between a thread's consecutive items
  // parameter sets per thread: with G = 32 the rows < 32 and >= 32 of a tile are different groups
  static constexpr int kSets = (G >= 64 || kIter == 1) ? 1 : 2;
  static_assert(kItems % NH == 0 && NH % kRI == 0, "thread count must tile the items");
  static_assert(kSets == 1 || (kIter % 2 == 0 && kRowStep * (kIter / 2) == 32), "two groups need an even split");

  uint32_t code[kQuant ? kIter : 1];
  float ps[kQuant ? kSets : 1][kPer], pz[kQuant ? kSets : 1][kPer];
  uint4 row[kQuant ? 1 : kIter];  // bf16 cache
};

struct RolePtrs {      // what distinguishes the K half from the V half
  const uint32_t* codes;  // packed tile base of (layer, head): row-major [Tcap rows][row dwords]
  const float* ps;        // parameter arrays of (layer, head)
  const float* pz;
  uint16_t* lds;          // first of the two LDS tiles of this role (the second follows it)
  bool is_v;
};

template <int BITS, int G, int NH>
__device__ __forceinline__ void fetch_cache_tile(Stage<BITS, G, NH>& st, const RolePtrs& rp, int Tcap, int tile, int u) {
  using S = Stage<BITS, G, NH>;
  constexpr int kRowDw = kD * BITS / 32;  // dwords per K row == dwords per V block row
  const uint32_t* base = rp.codes + (size_t)tile * kTile * kRowDw;
  if constexpr (!S::kQuant) {
#pragma unroll
    for (int it = 0; it < S::kIter; ++it) st.row[it] = reinterpret_cast<const uint4*>(base)[u + it * NH];
  } else {
#pragma unroll
    for (int it = 0; it < S::kIter; ++it) st.code[it] = base[u + it * NH];
    const int o = u % S::kRI;
#pragma unroll
    for (int set0 = 0; set0 < S::kSets; ++set0) {
      // 32-row half of the tile this set belongs to (a thread with a single item has a single row)
      const int set = (G >= 64) ? 0 : (S::kIter == 1 ? (u / S::kRI) / 32 : set0);
      // K: parameters [group][channel], the item's channels are o*kPer.. of group (tile, set)
      // V: parameters [token][channel group], the item's tokens are o*kPer.. of channel group `set`
      const float *ps, *pz;
      size_t stride;
      if (!rp.is_v) {
        const size_t g = (G >= kTile) ? (size_t)tile / (G / kTile) : (size_t)tile * (kTile / G) + set;
        ps = rp.ps + g * kD + o * S::kPer;
        pz = rp.pz + g * kD + o * S::kPer;
        stride = 1;
      } else {
        const size_t t0 = (size_t)tile * kTile + o * S::kPer;
        ps = rp.ps + t0 * (kD / G) + set;
        pz = rp.pz + t0 * (kD / G) + set;
        stride = kD / G;
      }
      if (!rp.is_v || kD / G == 1) {  // consecutive parameters: 16-byte loads (t0 and o * kPer are multiples of 8)
#pragma unroll
        for (int e = 0; e < S::kPer; e += 4) {
          const float4 a4 = *reinterpret_cast<const float4*>(ps + e), b4 = *reinterpret_cast<const float4*>(pz + e);
          st.ps[set0][e] = a4.x; st.ps[set0][e + 1] = a4.y; st.ps[set0][e + 2] = a4.z; st.ps[set0][e + 3] = a4.w;
          st.pz[set0][e] = b4.x; st.pz[set0][e + 1] = b4.y; st.pz[set0][e + 2] = b4.z; st.pz[set0][e + 3] = b4.w;
        }
      } else {
#pragma unroll
        for (int e = 0; e < S::kPer; ++e) {
          st.ps[set0][e] = ps[e * stride];
          st.pz[set0][e] = pz[e * stride];
        }
      }
    }
  }
}

template <int BITS, int G, int NH>
__device__ __forceinline__ void store_cache_tile(const Stage<BITS, G, NH>& st, uint16_t* lds, int u) {
  using S = Stage<BITS, G, NH>;
  const int r0 = u / S::kRI, o = u % S::kRI;
  // The cache's canonical view: (code - zero) exactly, ONE fp32 multiply by the scale, then bf16.
  // (A fused code * scale + (-zero * scale) would save an instruction per element, but it rounds
  // zero * scale first and so breaks ties differently: products of a small integer with
  // scale = range / levels land on bf16 midpoints often enough to move a dominant key's logit.)
#pragma unroll
  for (int it = 0; it < S::kIter; ++it) {
    uint16_t* dst = lds + (r0 + it * S::kRowStep) * kLdsStride + o * S::kPer;
    if constexpr (!S::kQuant) {
      *reinterpret_cast<uint4*>(dst) = st.row[it];
    } else {
      const int set = (S::kSets == 1) ? 0 : (it >= S::kIter / 2);
      float f[S::kPer];
      unpack_codes<BITS>(st.code[it], f);
      uint32_t pk[S::kPer / 2];
#pragma unroll
      for (int e = 0; e < S::kPer; e += 2)
        pk[e / 2] = pack_bf16((f[e] - st.pz[set][e]) * st.ps[set][e], (f[e + 1] - st.pz[set][e + 1]) * st.ps[set][e + 1]);
#pragma unroll
      for (int w = 0; w < S::kPer / 8; ++w)
        *reinterpret_cast<uint4*>(dst + w * 8) = make_uint4(pk[4 * w], pk[4 * w + 1], pk[4 * w + 2], pk[4 * w + 3]);
    }
  }
}

// Frame tiles (bf16 rows as given).  K half: 512 items of 16 bytes, item = (token i/8, channel run
// i%8), copied as they are.  V half: the tile must land transposed ([channel][token]); an item is
// (token octet, channel pair): eight 4-byte loads down the token axis (a wave's loads cover whole
// 128-byte rows), two byte-permutes per register pair, and two 16-byte LDS writes.
template <int NH>
struct FrameStage {
  static constexpr int kIterK = 512 / NH;  // 16-byte items per K thread
  static constexpr int kIterV = 256 / NH;  // 8-dword items per V thread
  static_assert(kIterK * 4 == kIterV * 8, "both roles stage the same number of registers");
  uint32_t w[kIterK * 4];
};

// Frame tile, V half: which (channel pair c2 = 0..31, token octet tq) thread u of the V half stages first (its
// further items are NH / 32 octets further down).  Eight consecutive lanes take four channel pairs of two
// octets, so that their 16-byte LDS writes - rows 2 * c2 (+1) of 144 bytes, column 16 * tq - fall into eight
// different bank groups; with consecutive channel pairs on consecutive lanes they would share four.
__device__ __forceinline__ void frame_v_item(int u, int& c2, int& tq) {
  const int l = u & 63, w = u >> 6;
  c2 = 4 * (l >> 3) + (l & 3);
  tq = 2 * w + ((l >> 2) & 1);
}

// The frame's rows are read through a buffer resource that covers exactly the n rows of the (layer, head): the
// loads take one 32-bit offset register that never changes plus a scalar offset per tile (no 64-bit address per
// load), and rows past the frame read as zeros by the resource's range check (their logits are masked, their
// values must be finite).
struct FrameRows {
  __amdgpu_buffer_rsrc_t rsrc;
  uint32_t row_bytes;  // stride between rows
  uint32_t voff;       // this thread's byte offset inside a tile
};

__device__ __forceinline__ FrameRows frame_rows(const uint16_t* xh, int64_t x_st, int n, bool is_v, int u) {
  FrameRows f;
  f.row_bytes = (uint32_t)x_st * 2u;
  const uint32_t bytes = ((uint32_t)(n - 1) * (uint32_t)x_st + (uint32_t)kD) * 2u;
  f.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(xh), 0, (int)bytes, 0x00020000);
  // K: item (token u/8, channels 8*(u%8)..);  V: item (token octet u/32, channel pair u%32)
  int c2, tq;
  frame_v_item(u, c2, tq);
  f.voff = is_v ? (uint32_t)(8 * tq) * f.row_bytes + 4u * c2 : (uint32_t)(u >> 3) * f.row_bytes + 16u * (u & 7);
  return f;
}

template <int NH>
__device__ __forceinline__ void fetch_frame_tile(FrameStage<NH>& st, const FrameRows& f, bool is_v, int tile) {
  using F = FrameStage<NH>;
  const uint32_t tile_off = (uint32_t)tile * kTile * f.row_bytes;  // scalar
  if (!is_v) {
#pragma unroll
    for (int it = 0; it < F::kIterK; ++it) {  // items u + it * NH: NH / 8 rows further down
      const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(f.rsrc, f.voff, tile_off + it * (NH / 8) * f.row_bytes, 0);
      st.w[4 * it] = v[0]; st.w[4 * it + 1] = v[1]; st.w[4 * it + 2] = v[2]; st.w[4 * it + 3] = v[3];
    }
  } else {
#pragma unroll
    for (int it = 0; it < F::kIterV; ++it) {  // items u + it * NH: NH / 32 token octets further down
#pragma unroll
      for (int e = 0; e < 8; ++e)
        st.w[8 * it + e] = __builtin_amdgcn_raw_buffer_load_b32(f.rsrc, f.voff, tile_off + (it * (NH / 32) * 8 + e) * f.row_bytes, 0);
    }
  }
}

template <int NH>
__device__ __forceinline__ void store_frame_tile(const FrameStage<NH>& st, uint16_t* lds, bool is_v, int u) {
  using F = FrameStage<NH>;
  if (!is_v) {
#pragma unroll
    for (int it = 0; it < F::kIterK; ++it) {
      const int i = u + it * NH;
      *reinterpret_cast<uint4*>(lds + (i >> 3) * kLdsStride + (i & 7) * 8) =
          make_uint4(st.w[4 * it], st.w[4 * it + 1], st.w[4 * it + 2], st.w[4 * it + 3]);
    }
  } else {
#pragma unroll
    for (int it = 0; it < F::kIterV; ++it) {
      int c2, tq;
      frame_v_item(u, c2, tq);
      tq += it * (NH / 32);
      uint32_t lo[4], hi[4];  // tokens 8tq.. of channel 2*c2 and of channel 2*c2+1
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        lo[k] = __builtin_amdgcn_perm(st.w[8 * it + 2 * k + 1], st.w[8 * it + 2 * k], 0x05040100u);
        hi[k] = __builtin_amdgcn_perm(st.w[8 * it + 2 * k + 1], st.w[8 * it + 2 * k], 0x07060302u);
      }
      *reinterpret_cast<uint4*>(lds + (2 * c2) * kLdsStride + 8 * tq) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
      *reinterpret_cast<uint4*>(lds + (2 * c2 + 1) * kLdsStride + 8 * tq) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
    }
  }
}

// "No vector-memory load is outstanding here" as an instruction (s_waitcnt vmcnt(0)).  A tile loop fetches the next
// tile under a condition and consumes it under the same condition further down; the compiler does not connect the
// two, assumes that fetched registers may still be in flight on the path that skips the consumer, and would then
// wait for ALL loads - the prefetch just issued included - in front of whatever reuses one of those registers in the
// next iteration or the next loop.  Stated at the end of an iteration, where it is true anyway, it costs nothing.
__device__ __forceinline__ void no_loads_in_flight() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// max of a value with the one held by the lane 32 apart (the other half of the same query's
// tokens): one v_permlane32_swap instead of a round trip through the LDS crossbar
__device__ __forceinline__ float xhalf_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// A callable that issues `N` MFMAs per call (the softmax block uses N to lay out its issue order).
template <int N, typename F>
struct MfmaHook {
  static constexpr int kMfma = N;
  F f;
  __device__ __forceinline__ void operator()(int i) const { f(i); }
};
template <int N, typename F>
__device__ __forceinline__ MfmaHook<N, F> with_mfma(F f) { return MfmaHook<N, F>{f}; }

// ---- partition of the (unit, tile) line over the workgroups -----------------------------------------
struct Partition {
  long long total;  // n_units * n_tiles
  int n_tiles, n_wgs;
  // 64-bit division is a long instruction sequence on this target; launches of realistic size fit 32 bits
  __host__ __device__ bool small() const { return total * (n_wgs + 1) < (1ll << 31); }
  __host__ __device__ long long begin(int w) const {
    return small() ? (long long)((unsigned)total * (unsigned)w / (unsigned)n_wgs) : total * w / n_wgs;
  }
  // workgroup whose piece holds item x
  __host__ __device__ int owner(long long x) const {
    return small() ? (int)((((unsigned)x + 1u) * (unsigned)n_wgs + (unsigned)total - 1u) / (unsigned)total) - 1
                   : (int)(((x + 1) * n_wgs + total - 1) / total) - 1;
  }
  __host__ __device__ int unit_of(long long x) const {
    return small() ? (int)((unsigned)x / (unsigned)n_tiles) : (int)(x / n_tiles);
  }
  __host__ __device__ int first_wg(int unit) const { return owner((long long)unit * n_tiles); }
  __host__ __device__ int last_wg(int unit) const { return owner((long long)(unit + 1) * n_tiles - 1); }
};

// ---- the kernel ----------------------------------------------------------------------------------
// ONE_LAYER: the launch works on a single layer (the per-layer calls).  The layer index is then a constant, so every
// pointer of the launch can be fetched from the kernel arguments right at the start, in one round trip, instead of
// after the workgroup has worked out which layer its piece belongs to.
template <int BITS, int G, int NW, int QB, bool ONE_LAYER>
__global__ __launch_bounds__(NW * 64) void attend_kernel(const AttendArgs a) {
  constexpr int NT = NW * 64, NH = NT / 2;
  constexpr int kRowsWG = 32 * QB * NW;  // query rows per workgroup
  {
    // The argument block is read field by field further down, each read a scalar load the next instructions wait
    // for, and at the start of a launch every one of them misses the scalar cache: several memory round trips in a
    // row before a workgroup can ask for its first tile.  One load from every 64-byte line the kernel will touch
    // (the fields behind the layer table, and the first layer's pointers), all issued here and waited for once,
    // brings those lines in together.
#if defined(__HIP_DEVICE_COMPILE__)  // (the builtin exists in the device pass only)
    const uint32_t* args = static_cast<const uint32_t*>(__builtin_amdgcn_kernarg_segment_ptr());
    constexpr unsigned kFirst = offsetof(AttendArgs, n_layers) / 4, kLast = (sizeof(AttendArgs) - 4) / 4;
    const uint32_t w0 = args[0], w1 = args[16], w2 = args[kFirst], w3 = args[kFirst + 16], w4 = args[kFirst + 32],
                   w5 = args[kLast];
    asm volatile("" ::"s"(w0), "s"(w1), "s"(w2), "s"(w3), "s"(w4), "s"(w5));
#endif
  }
  __shared__ __attribute__((aligned(16))) uint16_t lds_k[2][kLdsTile];
  __shared__ __attribute__((aligned(16))) uint16_t lds_v[2][kLdsTile];

  const int H = a.H, n = a.n, Tc = a.Tc;
  const int nqb = (n + kRowsWG - 1) / kRowsWG;
  // the wave index as a scalar the compiler knows to be the same for all lanes: what depends on it - the staging
  // role and every pointer chosen by it - lives in scalar registers, and the role's branches are scalar branches
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int j = lane & 31, hh = lane >> 5;
  const int krow = tau(j);
  const float c2 = a.qscale;  // softmax scale * log2(e): p = 2^(c2 * (logit - max))
  // staging role of this wave: first half of the workgroup's waves K, second half V
  const bool is_v = wave >= NW / 2;
  const int u = (is_v ? wave - NW / 2 : wave) * 64 + lane;

  // tiles of a unit: cache blocks, then the frame's own tokens (each range padded to 64 on its own)
  const int n_ct = (Tc + kTile - 1) / kTile, n_ft = (n + kTile - 1) / kTile;
  const Partition part{(long long)a.n_layers * H * nqb * (n_ct + n_ft), n_ct + n_ft, (int)gridDim.x};
  // Logical workgroup.  Workgroups whose blockIdx agree modulo 8 run on the same XCD and share its L2;
  // when every unit is cut into the same number of key ranges, the query blocks of one (layer, head,
  // key range) - which read the same K/V tiles - are placed on one XCD.
  // (Every integer division by a launch parameter is some thirty instructions here, and a workgroup's first tile
  // waits behind all of them: where the quotients are already at hand they are kept - `fast` below - instead of
  // being derived again from the logical index.)
  int wg = blockIdx.x;
  bool fast = false;      // this workgroup's (unit, range, query block, head) are known without further divisions
  int f_unit = 0, f_range = 0, f_qb = 0, f_head = 0;
  if (a.xcd_ranges > 0) {
    const int xcd = wg & 7, slot = wg >> 3;
    const int sq = slot / nqb, sr = slot - sq * nqb;
    const int g = sq * 8 + xcd;  // (layer, head, key range) triple
    const int gq = g / a.xcd_ranges, gr = g - gq * a.xcd_ranges;
    wg = (gq * nqb + sr) * a.xcd_ranges + gr;
    if (a.equal_ranges == a.xcd_ranges) {  // unit = wg / ranges, range = wg % ranges
      fast = true;
      f_unit = gq * nqb + sr;
      f_range = gr;
      f_qb = sr;      // unit % nqb
      f_head = gq;    // unit / nqb: (layer, head); the head itself when the launch has one layer
    }
  }
  // this workgroup's piece [piece_first, piece_end) of the (unit, tile) line: an equal share of the line, or - when
  // every unit is cut into the same ranges - range wg % R of unit wg / R from the host's table of range starts
  // (read with constant indices: a dynamically indexed kernel argument would be copied to scratch memory)
  long long piece_first, piece_end;
  int my_range = 0;  // which of its unit's key ranges this workgroup holds (equal ranges only)
  if (a.equal_ranges <= 0) {
    piece_first = part.begin(wg);
    piece_end = part.begin(wg + 1);
  } else {
    const int un = fast ? f_unit : wg / a.equal_ranges;
    my_range = fast ? f_range : wg - un * a.equal_ranges;
    int b0 = 0, b1 = 0;
#pragma unroll
    for (int i = 0; i < kMaxPieces; ++i) {
      if (i == my_range) { b0 = a.range_begin[i]; b1 = a.range_begin[i + 1]; }
    }
    piece_first = (long long)un * part.n_tiles + b0;
    piece_end = (long long)un * part.n_tiles + b1;
    if (!fast) f_unit = un;
  }

  for (long long pos = piece_first; pos < piece_end;) {
  // with equal ranges a piece lies inside one unit
  const int unit = a.equal_ranges > 0 ? f_unit : part.unit_of(pos);
  const int t_begin = (int)(pos - (long long)unit * part.n_tiles);
  const int t_end = (int)min((long long)part.n_tiles, t_begin + (piece_end - pos));
  pos += t_end - t_begin;
  int qb, h, lb;
  if (fast && ONE_LAYER) {
    qb = f_qb; h = f_head; lb = 0;
  } else {
    qb = unit % nqb;
    const int lh = unit / nqb;
    lb = ONE_LAYER ? 0 : lh / H;
    h = lh - lb * H;
  }
  const bool whole = t_begin == 0 && t_end == part.n_tiles;
  const int c_begin = min(t_begin, n_ct), c_end = min(t_end, n_ct);
  const int f_begin = max(t_begin, n_ct) - n_ct, f_end = max(t_end, n_ct) - n_ct;

  const AttendLayer& ly = a.layer[lb];
  const uint16_t* qh = ly.q + (size_t)h * a.q_sh;
  RolePtrs rp;
  rp.is_v = is_v;
  rp.codes = (is_v ? ly.vc : ly.kc) + (size_t)h * a.code_head;
  rp.ps = is_v ? ly.vs + (size_t)h * a.vparam_head : ly.ks + (size_t)h * a.kparam_head;
  rp.pz = is_v ? ly.vz + (size_t)h * a.vparam_head : ly.kz + (size_t)h * a.kparam_head;
  rp.lds = is_v ? lds_v[0] : lds_k[0];
  const uint16_t* xh = is_v ? ly.v + (size_t)h * a.v_sh : ly.k + (size_t)h * a.k_sh;
  const int64_t x_st = is_v ? a.v_st : a.k_st;

  // query fragments (B operand): lane holds channels 16*ks + 8*hh .. +8 of its query row, as given
  // (the softmax scale is applied to the fp32 logits, so no extra bf16 rounding enters)
  const int q_row0 = qb * kRowsWG + wave * 32 * QB;  // first row of this wave
  bf16x8 qf[QB][4];
#pragma unroll
  for (int cb = 0; cb < QB; ++cb) {
    const int q_row = q_row0 + 32 * cb + j;
    const uint16_t* qp = qh + (size_t)min(q_row, n - 1) * a.q_st;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      qf[cb][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qp + 16 * ks + 8 * hh));
  }
  // query blocks of this wave that hold at least one real row (wave-uniform)
  const int n_cb = q_row0 >= n ? 0 : min(QB, (n - q_row0 + 31) / 32);

  f32x16 o0[QB], o1[QB];
  // softmax state per query block: mc = -(reference of the exponent, log2 domain) so that a probability is
  // 2^(c2 * logit + mc), and this lane's share of the row sum
  float mc[QB], l[QB];
#pragma unroll
  for (int cb = 0; cb < QB; ++cb) {
#pragma unroll
    for (int r = 0; r < 16; ++r) { o0[cb][r] = 0.f; o1[cb][r] = 0.f; }
    mc[cb] = kNoReference;
    l[cb] = 0.f;
  }
  // softmax of one query block over the 32 tokens of a half-step: masks tokens >= valid, exponentiates into
  // packed bf16 and adds the row sums.  `hook(i)`, i = 0..3, is called before each quarter of the
  // exponentials: the caller issues MFMAs there, so that the matrix pipe works underneath this arithmetic.
  // The reference of the exponent is NOT the running row maximum: it stays where it is while the row sums
  // stay below 2^kSumLog2 - probabilities above 1 are as exact as those below, in bf16 as in fp32 - and no
  // maximum is computed at all on that path (half an instruction per logit saved).  Only when some row's sum
  // passes the limit (or, the first time, when there is no reference yet: every finite logit then
  // exponentiates to infinity) the block is redone the classical way: row maximum, new reference, sums and
  // accumulators rescaled, probabilities recomputed.  The MFMAs of the hook belong to other blocks and are
  // not repeated; this block's own PV product is issued by the caller after this function returns.
  auto softmax_half = [&](f32x16& sv, u32x4 (&pb)[2], float& mcr, float& lsum, f32x16& oa, f32x16& ob, int tok0,
                          int valid, auto&& hook) {
    if (valid < tok0 + 32) {  // tokens past the end of the cache / of the frame
      // (the limit passes through an opaque move so that the 16 compares stay inside this rarely
      // taken branch instead of being hoisted into every tile)
      int lim = valid - tok0;
      asm volatile("" : "+s"(lim));
      lim -= 8 * hh;
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (16 * (r >> 3) + (r & 7) >= lim) sv[r] = -INFINITY;
    }
    float psum = lsum;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      hook(q4);
#pragma unroll
      for (int r = 4 * q4; r < 4 * q4 + 4; r += 2) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[r], c2, mcr));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[r + 1], c2, mcr));
        const uint32_t w = pack_bf16(p0, p1);
        pb[r >> 3][(r >> 1) & 3] = w;  // registers r = 8*k2 .. 8*k2+7 are the B operand of token step k2
        // row sum of the ROUNDED probabilities (what the PV product sees): v_dot2c_f32_bf16
        psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), __builtin_bit_cast(bf16x2, 0x3f803f80u),
                                               psum, false);
      }
    }
    // prescribed issue order of this block, per quarter: its MFMAs spread between its 12 vector
    // instructions (4 fma, 4 exp, 2 convert, 2 dot) - the MFMAs execute while the VALU works
    constexpr int kMfmaPerQuarter = std::remove_reference_t<decltype(hook)>::kMfma;
    if constexpr (kMfmaPerQuarter > 0) {
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        // masks: 0x008 MFMA, 0x002 VALU (without transcendentals), 0x400 transcendental
        if constexpr (kMfmaPerQuarter == 2) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
          __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
        } else {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
          __builtin_amdgcn_sched_group_barrier(0x400, 4, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
        }
      }
    }
    if (__builtin_expect(__any(!(psum <= kSumLimit)), 0)) {  // some row sum passed the limit (or is not finite): redo with a new reference
      float mx = fmaxf(fmaxf(sv[0], sv[1]), sv[2]);  // v_max3 chain
#pragma unroll
      for (int r = 3; r < 15; r += 2) mx = fmaxf(fmaxf(mx, sv[r]), sv[r + 1]);
      mx = xhalf_max(fmaxf(mx, sv[15]));  // both lane halves of a row agree on it
      // new reference = max(old, row maximum of this half-step) in the log2 domain; rows whose tokens are all
      // masked here keep theirs
      const float ref_old = -mcr;
      const float ref_new = fmaxf(ref_old, mx * c2);
      const float alpha = __builtin_amdgcn_exp2f(ref_old - ref_new);  // 0 the first time (no reference yet)
      lsum *= alpha;
#pragma unroll
      for (int r = 0; r < 16; ++r) { oa[r] *= alpha; ob[r] *= alpha; }
      mcr = -ref_new;
      psum = lsum;
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[r], c2, mcr));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[r + 1], c2, mcr));
        const uint32_t w = pack_bf16(p0, p1);
        pb[r >> 3][(r >> 1) & 3] = w;
        psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), __builtin_bit_cast(bf16x2, 0x3f803f80u),
                                               psum, false);
      }
    }
    // keep this block's probabilities in this block (the compiler would otherwise sink the
    // exponentials down to their consumer, next to the MFMAs they are meant to overlap with)
    asm volatile("" : "+v"(pb[0]), "+v"(pb[1]));
    lsum = psum;
  };

  // one tile of 64 tokens held in LDS buffer `buf`, of which the first `valid` are real
  auto compute = [&](int buf, int valid) {
    if (n_cb == 0) return;
    const uint16_t* lk = lds_k[buf] + krow * kLdsStride + 8 * hh;
    const uint16_t* lv = lds_v[buf] + j * kLdsStride + 8 * hh;
    auto load_k = [&](bf16x8 (&kf)[4], int half) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) kf[ks] = *reinterpret_cast<const bf16x8*>(lk + 32 * half * kLdsStride + 16 * ks);
    };
    auto load_v = [&](bf16x8 (&vf)[2][2], int half) {
#pragma unroll
      for (int k2 = 0; k2 < 2; ++k2) {
        vf[k2][0] = *reinterpret_cast<const bf16x8*>(lv + 32 * half + 16 * k2);
        vf[k2][1] = *reinterpret_cast<const bf16x8*>(lv + 32 * kLdsStride + 32 * half + 16 * k2);
      }
    };
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // step i (0..3) of S^T = K Q^T for one query block (contraction over 16 channels per step)
    auto qk_step = [&](f32x16& sv, const bf16x8 (&kf)[4], int cb, int i) {
      sv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i], qf[cb][i], i == 0 ? zero : sv, 0, 0, 0);
    };
    // step i (0..3) of O^T += V^T P^T for one query block: token step i/2, channel half i%2
    auto pv_step = [&](int cb, const bf16x8 (&vf)[2][2], const u32x4 (&pb)[2], int i) {
      const int k2 = i >> 1;
      const bf16x8 p = __builtin_bit_cast(bf16x8, pb[k2]);
      if (i & 1) o1[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[k2][1], p, o1[cb], 0, 0, 0);
      else o0[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[k2][0], p, o0[cb], 0, 0, 0);
    };

    if constexpr (QB == 2) {
      // Software pipeline over the two half-steps and the two query blocks A, B of the wave: every
      // block of softmax arithmetic has independent MFMAs issued inside it —
      //   SM(A,h):  S(B,h) [and O(B,h-1)]      SM(B,h):  O(A,h) [and S(A,h+1)]
      // Blocks past the end of the frame are computed on clamped rows and never stored.
      bf16x8 kf[4], vf[2][2];
      f32x16 sA, sB;
      u32x4 pA[2], pB[2];
      load_k(kf, 0);
#pragma unroll
      for (int i = 0; i < 4; ++i) qk_step(sA, kf, 0, i);
      load_v(vf, 0);
      // ---- half 0 ----
      // (wave priority falls as a wave advances through a tile: of the two waves that share a SIMD the one that is
      // behind is served first, so they stay within a block of each other and each one's MFMAs run under the
      // other's softmax arithmetic, instead of the older wave finishing its tile first and the younger one
      // then working through its own alone; measured 2.7 % on the kernel)
      __builtin_amdgcn_s_setprio(3);
      softmax_half(sA, pA, mc[0], l[0], o0[0], o1[0], 0, valid, with_mfma<1>([&](int i) { qk_step(sB, kf, 1, i); }));
      load_k(kf, 1);
      __builtin_amdgcn_s_setprio(2);
      softmax_half(sB, pB, mc[1], l[1], o0[1], o1[1], 0, valid, with_mfma<2>([&](int i) {
        pv_step(0, vf, pA, i);
        qk_step(sA, kf, 0, i);
      }));
      // ---- half 1 ----
      __builtin_amdgcn_s_setprio(1);
      softmax_half(sA, pA, mc[0], l[0], o0[0], o1[0], 32, valid, with_mfma<2>([&](int i) {
        pv_step(1, vf, pB, i);
        qk_step(sB, kf, 1, i);
      }));
      load_v(vf, 1);
      __builtin_amdgcn_s_setprio(0);
      softmax_half(sB, pB, mc[1], l[1], o0[1], o1[1], 32, valid, with_mfma<1>([&](int i) { pv_step(0, vf, pA, i); }));
#pragma unroll
      for (int i = 0; i < 4; ++i) pv_step(1, vf, pB, i);
    } else {
      bf16x8 kf[4], vf[2][2];
      load_k(kf, 0);
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        if (32 * half >= valid) break;
        f32x16 sv;
#pragma unroll
        for (int i = 0; i < 4; ++i) qk_step(sv, kf, 0, i);
        load_v(vf, half);
        if (half == 0 && valid > 32) load_k(kf, 1);
        u32x4 pw[2];
        softmax_half(sv, pw, mc[0], l[0], o0[0], o1[0], 32 * half, valid, with_mfma<0>([](int) {}));
#pragma unroll
        for (int i = 0; i < 4; ++i) pv_step(0, vf, pw, i);
      }
    }
  };
  // Phase 1: this range's tiles of the packed cache; phase 2: its tiles of the frame.  Each phase is
  // software pipelined on its own: a tile is fetched into registers while an earlier one is
  // computed, then converted into a free LDS buffer.
  // the previous unit's last tile has been read by everybody (a workgroup's first unit has nothing to wait for, and a
  // barrier there would only make its waves wait for the last of them to be started)
  if (pos - (t_end - t_begin) != piece_first) __syncthreads();
  int cur = 0;      // two LDS buffers, one barrier per tile
  if (c_begin < c_end) {
    Stage<BITS, G, NH> st;
    fetch_cache_tile<BITS, G, NH>(st, rp, a.Tcap, c_begin, u);
    store_cache_tile<BITS, G, NH>(st, rp.lds + cur * kLdsTile, u);
    no_loads_in_flight();
    for (int t = c_begin; t < c_end; ++t) {
      __syncthreads();  // tile t is in lds[cur]; everybody is done reading lds[cur^1]
      if (t + 1 < c_end) fetch_cache_tile<BITS, G, NH>(st, rp, a.Tcap, t + 1, u);
      compute(cur, min(kTile, Tc - t * kTile));
      if (t + 1 < c_end) store_cache_tile<BITS, G, NH>(st, rp.lds + (cur ^ 1) * kLdsTile, u);
      no_loads_in_flight();
      cur ^= 1;
    }
  }
  if (f_begin < f_end) {
    FrameStage<NH> st;
    const FrameRows fr = frame_rows(xh, x_st, n, is_v, u);
    fetch_frame_tile<NH>(st, fr, is_v, f_begin);
    store_frame_tile<NH>(st, rp.lds + cur * kLdsTile, is_v, u);  // lds[cur] was last read two barriers ago
    no_loads_in_flight();
    for (int t = f_begin; t < f_end; ++t) {
      __syncthreads();
      if (t + 1 < f_end) fetch_frame_tile<NH>(st, fr, is_v, t + 1);
      compute(cur, min(kTile, n - t * kTile));
      if (t + 1 < f_end) store_frame_tile<NH>(st, rp.lds + (cur ^ 1) * kLdsTile, is_v, u);
      no_loads_in_flight();
      cur ^= 1;
    }
  }

  // accumulator register r of o0 (o1) is channel 8*(r/4) + 4*hh + r%4 (+32) of the lane's query row
#pragma unroll
  for (int cb = 0; cb < QB; ++cb) {
    const int q_row = q_row0 + 32 * cb + j;
    const float lsum = l[cb] + __shfl_xor(l[cb], 32);  // the two lane halves saw disjoint tokens
    if (q_row >= n) continue;  // (both lanes of a row leave together, so the lane exchange below stays paired)
    if (whole) {
      const float inv = 1.0f / lsum;
      uint16_t* op = ly.out + ((size_t)h * n + q_row) * kD;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int c = 8 * q4 + 4 * hh;
        *reinterpret_cast<uint2*>(op + c) = make_uint2(pack_bf16(o0[cb][4 * q4] * inv, o0[cb][4 * q4 + 1] * inv),
                                                       pack_bf16(o0[cb][4 * q4 + 2] * inv, o0[cb][4 * q4 + 3] * inv));
        *reinterpret_cast<uint2*>(op + 32 + c) = make_uint2(pack_bf16(o1[cb][4 * q4] * inv, o1[cb][4 * q4 + 1] * inv),
                                                            pack_bf16(o1[cb][4 * q4 + 2] * inv, o1[cb][4 * q4 + 3] * inv));
      }
    } else {
      // Partial of a cut unit, as fp16 mantissas under one power-of-two scale per query row (the
      // row's largest magnitude maps into [0.5, 1): 11 bits below the row maximum, half the bytes of
      // fp32).  Lane (j, hh) owns 32 channels of row j, in register order o0[0..15], o1[0..15], as
      // four 16-byte pieces i; a block of 32 rows is stored [i][hh][j], so that every store
      // instruction of the wave covers 1 KB of consecutive memory.
      const int piece = a.equal_ranges > 0 ? my_range : wg - part.first_wg(unit);
      const int nblk = (n + 31) / 32;
      const size_t row = (((size_t)piece * a.n_layers + lb) * H + h) * n + q_row;
      const size_t blk = (((size_t)piece * a.n_layers + lb) * H + h) * nblk + (q_row >> 5);
      float amax = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) amax = fmaxf(amax, fmaxf(fabsf(o0[cb][r]), fabsf(o1[cb][r])));
      amax = xhalf_max(amax);
      const int e = __builtin_amdgcn_frexp_expf(amax);  // amax = f * 2^e, f in [0.5, 1)  (0 for amax == 0)
      uint32_t hw[16];
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        hw[r >> 1] = pack_f16(__builtin_amdgcn_ldexpf(o0[cb][r], -e), __builtin_amdgcn_ldexpf(o0[cb][r + 1], -e));
        hw[8 + (r >> 1)] = pack_f16(__builtin_amdgcn_ldexpf(o1[cb][r], -e), __builtin_amdgcn_ldexpf(o1[cb][r + 1], -e));
      }
      uint4* op = reinterpret_cast<uint4*>(a.attn_o) + blk * 256 + hh * 32 + j;
#pragma unroll
      for (int i = 0; i < 4; ++i) op[i * 64] = make_uint4(hw[4 * i], hw[4 * i + 1], hw[4 * i + 2], hw[4 * i + 3]);
      if (hh == 0)
        *reinterpret_cast<float4*>(a.attn_ml + row * 4) = make_float4(-mc[cb], lsum, __builtin_amdgcn_ldexpf(1.0f, e), 0.f);
    }
  }
  }  // units of this workgroup's piece

}

// Merge of the pieces of every unit that was cut:  out = sum_p 2^(m_p - M) O_p / sum_p 2^(m_p - M) l_p.
// (A separate launch on purpose: a device-wide release/acquire inside the attention kernel costs an
// L2 write-back per workgroup on this multi-die part, far more than a second small kernel.)
// Grid: y = chunk of 32 query rows of a unit; x = the unit when all units are cut alike, else a boundary
// between workgroups w-1 | w of the attention grid (w = blockIdx.x + 1), standing for the unit it falls
// into: a unit with several boundaries is handled at its first one, and a boundary that coincides with
// a unit's edge has nothing to merge.
// Thread = (row, lane half hh, quarter of the lane's 32 values): 8 fp16 values of every piece.
__global__ __launch_bounds__(256) void combine_kernel(const AttendArgs a) {
  // the merge shares its compute units with the chain's kernels of the same layer, which nothing waits for: its
  // waves are served first
  __builtin_amdgcn_s_setprio(3);
  const int H = a.H, n = a.n;
  const int nqb = (n + a.rows_wg - 1) / a.rows_wg;
  const int n_tiles = (a.Tc + kTile - 1) / kTile + (n + kTile - 1) / kTile;
  const Partition part{(long long)a.n_layers * H * nqb * n_tiles, n_tiles, a.n_wgs};
  int unit, S;
  if (a.equal_ranges > 0) {  // every unit is cut into the same number of ranges: x = unit
    unit = blockIdx.x;
    S = a.equal_ranges;
  } else {
    const int w = blockIdx.x + 1;
    const long long pos = part.begin(w);
    unit = part.unit_of(pos);
    if (pos == (long long)unit * n_tiles) return;
    const int w0 = part.first_wg(unit);
    if (w0 + 1 != w) return;
    S = part.last_wg(unit) - w0 + 1;
  }
  const int qb = unit % nqb, h = (unit / nqb) % H, lb = unit / (nqb * H);
  const int tid = threadIdx.x;
  const int jrow = tid & 31, hh = (tid >> 5) & 1, qd = tid >> 6;  // consecutive threads read consecutive 16-byte pieces
  const int q_row = qb * a.rows_wg + 32 * blockIdx.y + jrow;
  if (q_row >= n) return;
  const int nblk = (n + 31) / 32;
  const size_t rows = (size_t)a.n_layers * H * n, blks = (size_t)a.n_layers * H * nblk;
  const size_t row = ((size_t)lb * H + h) * n + q_row;
  const size_t blk = ((size_t)lb * H + h) * nblk + (q_row >> 5);
  float ms[kMaxPieces], ls[kMaxPieces], sc[kMaxPieces];
  float M = kNegBig;
#pragma unroll 4
  for (int s = 0; s < S; ++s) {
    const float4 ml = *reinterpret_cast<const float4*>(a.attn_ml + (s * rows + row) * 4);
    ms[s] = ml.x;
    ls[s] = ml.y;
    sc[s] = ml.z;
    M = fmaxf(M, ml.x);
  }
  float L = 0.f, acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
  for (int s = 0; s < S; ++s) {
    const float wgt = __builtin_amdgcn_exp2f(ms[s] - M);
    const uint4 o = reinterpret_cast<const uint4*>(a.attn_o)[(s * blks + blk) * 256 + qd * 64 + hh * 32 + jrow];
    L += wgt * ls[s];
    const float ws = wgt * sc[s];
    const uint32_t ow[4] = {o.x, o.y, o.z, o.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const f16x2 v = __builtin_bit_cast(f16x2, ow[i]);
      acc[2 * i] += ws * (float)v[0];
      acc[2 * i + 1] += ws * (float)v[1];
    }
  }
  const float inv = 1.0f / L;
  // values 8*qd + t of the lane: accumulator registers r = 8*(qd%2) + t of o0 (qd < 2) or o1, i.e.
  // channels 32*(qd/2) + 16*(qd%2) + {0, 8} + 4*hh + 0..3
  uint16_t* op = a.layer[lb].out + ((size_t)h * n + q_row) * kD + 32 * (qd >> 1) + 16 * (qd & 1) + 4 * hh;
  *reinterpret_cast<uint2*>(op) = make_uint2(pack_bf16(acc[0] * inv, acc[1] * inv), pack_bf16(acc[2] * inv, acc[3] * inv));
  *reinterpret_cast<uint2*>(op + 8) = make_uint2(pack_bf16(acc[4] * inv, acc[5] * inv), pack_bf16(acc[6] * inv, acc[7] * inv));
}

template <int BITS, int G, int NW, int QB>
static hipError_t launch_attend_t(const AttendArgs& a, hipStream_t stream, hipEvent_t between) {
  if (a.n_layers == 1) hipLaunchKernelGGL((attend_kernel<BITS, G, NW, QB, true>), dim3(a.n_wgs), dim3(NW * 64), 0, stream, a);
  else hipLaunchKernelGGL((attend_kernel<BITS, G, NW, QB, false>), dim3(a.n_wgs), dim3(NW * 64), 0, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (between && (e = hipEventRecord(between, stream)) != hipSuccess) return e;
  if (a.cut) {
    const int n_units = a.n_layers * a.H * ((a.n + a.rows_wg - 1) / a.rows_wg);
    hipLaunchKernelGGL(combine_kernel, dim3(a.equal_ranges > 0 ? n_units : a.n_wgs - 1, (a.rows_wg + 31) / 32), dim3(256), 0,
                       stream, a);
    e = hipGetLastError();
  }
  return e;
}

template <int BITS, int G>
static hipError_t launch_attend_v(const AttendArgs& a, hipStream_t stream, hipEvent_t between) {
  switch (a.variant) {
    case 1: return launch_attend_t<BITS, G, 4, 1>(a, stream, between);
    case 2: return launch_attend_t<BITS, G, 8, 1>(a, stream, between);
    case 3: return launch_attend_t<BITS, G, 8, 2>(a, stream, between);
    default: return launch_attend_t<BITS, G, 4, 2>(a, stream, between);
  }
}

// Host-side queries of the partition the kernel uses when the units are not all cut alike (for tests).
void partition_query(long long n_units, int n_tiles, int n_wgs, int wg, long long* begin, long long* end) {
  const Partition part{n_units * n_tiles, n_tiles, n_wgs};
  *begin = part.begin(wg);
  *end = part.begin(wg + 1);
}
void partition_unit_query(long long n_units, int n_tiles, int n_wgs, int unit, int* first_wg, int* last_wg) {
  const Partition part{n_units * n_tiles, n_tiles, n_wgs};
  *first_wg = part.first_wg(unit);
  *last_wg = part.last_wg(unit);
}

int attend_rows_per_workgroup(int variant) {
  return variant == 1 ? 128 : (variant == 3 ? 512 : 256);
}

AttendPlan plan_attend(int variant, int n_layers, int H, int n, int Tc, int want_wgs, size_t part_rows) {
  const int rows_wg = attend_rows_per_workgroup(variant);
  const int nqb = (n + rows_wg - 1) / rows_wg;
  const int n_units = n_layers * H * nqb;
  const int n_tiles = (Tc + kTile - 1) / kTile + (n + kTile - 1) / kTile;
  const long long total = (long long)n_units * n_tiles;
  // a piece never shorter than 4 tiles (unless a whole unit is), never more workgroups than items
  long long w = std::max<long long>(1, std::min<long long>(want_wgs, std::max<long long>(n_units, total / 4)));
  // the partial workspace holds `fit` pieces of every row, the merge at most kMaxPieces
  const int fit = (int)std::min<size_t>(kMaxPieces, part_rows / ((size_t)n_layers * H * ((n + 31) / 32 * 32)));
  AttendPlan p{};
  for (;; --w) {
    const Partition part{total, n_tiles, (int)w};
    int worst = 1;
    for (int unit = 0; unit < n_units; ++unit) worst = std::max(worst, part.last_wg(unit) - part.first_wg(unit) + 1);
    if (worst <= fit || w == 1) {
      p.n_wgs = (int)w;
      p.rows_wg = rows_wg;
      p.max_pieces = worst;
      return p;
    }
    if (w > n_units) w = std::max<long long>(n_units + 1, w - w / 8);  // then --w
  }
}

hipError_t launch_attend(const AttendArgs& a, hipStream_t stream, hipEvent_t between) {
  const int bits = a.bits, G = a.G;
  if (bits == 16) return launch_attend_v<16, 64>(a, stream, between);
  if (bits == 4 && G == 64) return launch_attend_v<4, 64>(a, stream, between);
  if (bits == 4 && G == 32) return launch_attend_v<4, 32>(a, stream, between);
  if (bits == 2 && G == 64) return launch_attend_v<2, 64>(a, stream, between);
  if (bits == 2 && G == 32) return launch_attend_v<2, 32>(a, stream, between);
  return hipErrorInvalidValue;
}

}  // namespace xsv
