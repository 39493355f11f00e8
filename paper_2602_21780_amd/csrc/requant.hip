// Gather by the keep list + dimension-adaptive quantization of the whole retained cache
// (paper Sec. 3.3: keys per channel over groups of G kept tokens, values per token over groups of G
// channels), and the canonical unpack used by export and by the stateless entry points.  gfx950.
//
// requant_kernel: one workgroup per (block of 64 new cache positions, head, layer), 256 threads,
// thread = (token tid/4 of the block, channel quarter tid%4 = 16 channels).
//   source row of a new position = keep[pos]: a cached token (read through its dequantized bf16
//   view (code - zero) * scale) or a row of the current frame (bf16 as given);
//   keys:   the 64x64 tile goes through LDS once for the per-channel min/max over the group's
//           tokens; codes are packed 16 channels per thread and written as coalesced 8-byte pieces;
//   values: min/max over a token's channel group by wave shuffles; the codes are transposed
//           through an LDS byte tile so the packed block is written [channel][token], the layout
//           the attention kernel's PV product consumes.
//   Writes go to the layer's OTHER buffer, so nothing is updated in place - except in a cache that is never pruned
//   (one buffer): there no row ever moves, a block is read and rewritten by its one workgroup, reads first.
//   Blocks whose rows stay where they are (the first frame's, or every block of old rows while nothing is pruned) are
//   re-quantized from their own dequantized values like everything else, but that reaches a fixed point after a
//   round or two; the step that sees a block come out bit-identical flags it, and from then on it is skipped: both
//   buffers hold it and re-quantizing it can only reproduce it.
// HBM-bound: every retained element is read once (packed) and written once (packed).
// Compiled with -ffp-contract=off; division is IEEE, rounding is nearest-even (rintf).
#include "xsv_internal.h"

namespace xsv {

__device__ __forceinline__ float round_bf16(float x) { return (float)(__bf16)x; }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ uint16_t bf16_bits(float x) { return __builtin_bit_cast(unsigned short, (__bf16)x); }

struct QParam {
  float s, z;
  float y;    // 1 / s, correctly rounded
  bool safe;  // the division-free quotient below may be used for this group
};

__device__ __forceinline__ QParam group_param(float lo, float hi, int bits) {
  const float levels = (float)((1 << bits) - 1);
  float s = (hi - lo) / levels;
  if (s == 0.0f) s = 1.0f;
  QParam p;
  p.s = s;
  p.z = rintf(-lo / s);
  p.y = 1.0f / s;
  // magnitudes for which no intermediate of exact_quotient over- or underflows in a way that could
  // change rint(x / s); anything else (also NaN) takes the division
  constexpr float kBig = 0x1p60f, kSmall = 0x1p-60f;
  p.safe = s >= kSmall && s <= kBig && fmaxf(fabsf(lo), fabsf(hi)) <= kBig;
  return p;
}

// x / s rounded to nearest, bit for bit the IEEE quotient, from y = RN(1 / s) and four fused multiply-adds
// instead of the eleven-instruction division sequence.  q0 = RN(x y) is within 2 ulp of x / s; the first
// correction with the remainder r = x - q s makes it faithful (within 1 ulp), and for a faithful q and a
// correctly rounded reciprocal RN(q + r y) is the correctly rounded quotient (Markstein's theorem; the
// remainder of a faithful quotient is exact in one FMA).  For |x / s| < 1/2 the low intermediates may lose
// bits to underflow, which cannot move rint() of the result off zero.
__device__ __forceinline__ float exact_quotient(float x, float s, float y) {
  float q = x * y;
  float r = __builtin_fmaf(-q, s, x);
  q = __builtin_fmaf(r, y, q);
  r = __builtin_fmaf(-q, s, x);
  return __builtin_fmaf(r, y, q);
}

__device__ __forceinline__ uint32_t quant_code_fast(float x, float s, float y, float z, int bits) {
  const float hi = (float)((1 << bits) - 1);
  float q = rintf(exact_quotient(x, s, y)) + z;
  q = fminf(fmaxf(q, 0.0f), hi);
  return (uint32_t)q;
}

__device__ __forceinline__ uint32_t quant_code(float x, float s, float z, int bits) {
  const float hi = (float)((1 << bits) - 1);
  float q = rintf(x / s) + z;
  q = fminf(fmaxf(q, 0.0f), hi);
  return (uint32_t)q;
}

// CARRY: RequantArgs::carry_values as a compile-time property (the default path carries no trace of the variant)
template <int BITS, int G, bool CARRY = false>
__global__ __launch_bounds__(256) void requant_kernel(const RequantArgs a) {
  constexpr bool kQuant = BITS != 16;
  constexpr int kRowDw = kD * BITS / 32;  // dwords per packed key row / value block row
  constexpr int kPer = kQuant ? 32 / BITS : 2;  // elements per dword
  constexpr uint32_t kMask = kQuant ? (1u << (BITS & 15)) - 1u : 0xffffu;
  constexpr int kKGroups = kTile / G;  // key groups per block of 64 tokens (1 or 2)
  constexpr int kVGroups = kD / G;     // value groups per token (1 or 2)

  __shared__ float xk[kTile][kD + 1];
  __shared__ float red_lo[4][kD], red_hi[4][kD];
  __shared__ float gs[2][kD], gz[2][kD], gy[2][kD];
  __shared__ int k_unsafe;  // some key group of this block needs the division
  __shared__ __attribute__((aligned(16))) uint16_t vt[kD][kTile + 8];  // value codes (or bf16), [channel][token]

  const int u = blockIdx.x, h = blockIdx.y, lb = blockIdx.z;
  const int tid = threadIdx.x, r = tid >> 2, cq = tid & 3;
  const int Tc = a.Tc, Tn = a.Tn, Tcap = a.pool.Tcap;
  const int layer = a.b.layer0 + lb;
  const int sb = a.b.src_buf(lb);
  const LayerCache src = layer_cache(a.pool, sb, layer);
  const LayerCache dst = layer_cache(a.pool, a.pool.buffers == 1 ? sb : sb ^ 1, layer);
  const int32_t* keep = a.ws.keep + list_index(a.ws.sets, layer, h) * a.ws.scores_stride;
  const int nv = min(kTile, Tn - u * kTile);  // valid new positions in this block

  // A block that holds the same cached rows as before the step and has already reproduced itself is final.
  const bool candidate = u < a.stable_blocks;  // the same for the whole workgroup
  uint8_t* const stable = a.stable_flag + ((size_t)layer * a.pool.H + h) * (Tcap / kTile) + u;
  if (candidate && *stable) return;
  unsigned changed = 0;  // candidate blocks: some code or parameter written differs from what was read

  if (tid == 0) k_unsafe = 0;  // (ordered before its readers and writers by the barriers of the key phase)
  // source row: arithmetic where the keep list is known without reading it (no dependent load in front of the gather)
  const int pos = u * kTile + r;
  int s_row = -1;
  if (r < nv) s_row = pos < a.identity_end ? pos : (pos >= Tn - a.n ? pos - (Tn - a.n) + Tc : keep[pos]);
  const bool row_valid = s_row >= 0;
  const bool from_cache = row_valid && s_row < Tc;

  // token ids travel with the rows (one copy per index set: head 0 writes the shared one)
  if ((h == 0 || a.ws.sets > 1) && cq == 0 && row_valid) {
    const size_t row0 = a.ws.sets > 1 ? (size_t)h * Tcap : 0;
    dst.tok_frame[row0 + pos] = from_cache ? src.tok_frame[row0 + s_row] : a.frame_id;
    dst.tok_index[row0 + pos] = from_cache ? src.tok_index[row0 + s_row] : s_row - Tc;
  }

  // values: all loads are issued here, ahead of the key phase, so that the kernel pays one memory
  // round trip for both; vraw = 16 gathered dwords (cache) or the 8 dwords of the frame row
  uint32_t vraw[16];
  float v_ps = 0.f, v_pz = 0.f;
  int v_shift = 0;
#pragma unroll
  for (int e = 0; e < 16; ++e) vraw[e] = 0u;
  if (from_cache) {
    const int blk = s_row / kTile, col = s_row % kTile;
    if constexpr (kQuant) {
      const uint32_t* rows = reinterpret_cast<const uint32_t*>(src.vc) + ((size_t)h * Tcap + (size_t)blk * kTile) * kRowDw + col / kPer;
      v_shift = (col % kPer) * BITS;
      const int vg = (cq * 16) / G;
      v_ps = src.vs[((size_t)h * Tcap + s_row) * kVGroups + vg];
      v_pz = src.vz[((size_t)h * Tcap + s_row) * kVGroups + vg];
#pragma unroll
      for (int e = 0; e < 16; ++e) vraw[e] = rows[(size_t)(cq * 16 + e) * kRowDw];
    } else {
      const uint16_t* rows = reinterpret_cast<const uint16_t*>(src.vc) + ((size_t)h * Tcap + (size_t)blk * kTile) * kD + col;
#pragma unroll
      for (int e = 0; e < 16; ++e) vraw[e] = rows[(size_t)(cq * 16 + e) * kD];
    }
  } else if (row_valid) {
    const uint4* p = reinterpret_cast<const uint4*>(a.b.v[lb] + (size_t)h * a.b.v_sh + (size_t)(s_row - Tc) * a.b.v_st + cq * 16);
    const uint4 v0 = p[0], v1 = p[1];
    vraw[0] = v0.x; vraw[1] = v0.y; vraw[2] = v0.z; vraw[3] = v0.w;
    vraw[4] = v1.x; vraw[5] = v1.y; vraw[6] = v1.z; vraw[7] = v1.w;
  }

  // ---------------- keys ----------------
  float x[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) x[e] = 0.f;
  uint32_t k_in[kQuant ? kRowDw / 4 : 1] = {};  // the row's packed key codes as read (candidate blocks compare against them)
  if (from_cache) {
    if constexpr (kQuant) {
      const uint32_t* codes = reinterpret_cast<const uint32_t*>(src.kc) + ((size_t)h * Tcap + s_row) * kRowDw + cq * (kRowDw / 4);
      const float* ks = src.ks + ((size_t)h * (Tcap / G) + s_row / G) * kD + cq * 16;
      const float* kz = src.kz + ((size_t)h * (Tcap / G) + s_row / G) * kD + cq * 16;
      uint32_t w[kRowDw / 4];
#pragma unroll
      for (int i = 0; i < kRowDw / 4; ++i) w[i] = k_in[i] = codes[i];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const uint32_t code = (w[e / kPer] >> ((e % kPer) * BITS)) & kMask;
        x[e] = round_bf16(((float)code - kz[e]) * ks[e]);
      }
    } else {
      const uint4* p = reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(src.kc) + ((size_t)h * Tcap + s_row) * kD + cq * 16);
      const uint4 v0 = p[0], v1 = p[1];
      const uint32_t ww[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) { x[2 * e] = bf16_lo(ww[e]); x[2 * e + 1] = bf16_hi(ww[e]); }
    }
  } else if (row_valid) {
    const uint4* p = reinterpret_cast<const uint4*>(a.b.k[lb] + (size_t)h * a.b.k_sh + (size_t)(s_row - Tc) * a.b.k_st + cq * 16);
    const uint4 v0 = p[0], v1 = p[1];
    const uint32_t ww[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) { x[2 * e] = bf16_lo(ww[e]); x[2 * e + 1] = bf16_hi(ww[e]); }
  }

  if constexpr (kQuant) {
#pragma unroll
    for (int e = 0; e < 16; ++e) xk[r][cq * 16 + e] = x[e];
    __syncthreads();
    {  // per-channel min/max: thread = (channel tid%64, 16-row part tid/64)
      const int c = tid & 63, part = tid >> 6;
      float lo = INFINITY, hi = -INFINITY;
      for (int i = part * 16; i < min(nv, part * 16 + 16); ++i) {
        lo = fminf(lo, xk[i][c]);
        hi = fmaxf(hi, xk[i][c]);
      }
      red_lo[part][c] = lo;
      red_hi[part][c] = hi;
    }
    __syncthreads();
    if (tid < kKGroups * kD) {
      const int c = tid & 63, gi = tid >> 6;
      constexpr int parts = 4 / kKGroups;  // 16-row parts per group
      if (gi * G < nv) {
        float lo = red_lo[gi * parts][c], hi = red_hi[gi * parts][c];
#pragma unroll
        for (int p = 1; p < parts; ++p) {
          lo = fminf(lo, red_lo[gi * parts + p][c]);
          hi = fmaxf(hi, red_hi[gi * parts + p][c]);
        }
        const QParam q = group_param(lo, hi, BITS);
        gs[gi][c] = q.s;
        gz[gi][c] = q.z;
        gy[gi][c] = q.y;
        if (!q.safe) k_unsafe = 1;
        const size_t gidx = ((size_t)h * (Tcap / G) + (size_t)u * kKGroups + gi) * kD + c;
        if (candidate) changed |= (__float_as_uint(src.ks[gidx]) ^ __float_as_uint(q.s)) | (__float_as_uint(src.kz[gidx]) ^ __float_as_uint(q.z));
        dst.ks[gidx] = q.s;
        dst.kz[gidx] = q.z;
      }
    }
    __syncthreads();
    if (row_valid) {
      const int gi = r / G;
      uint32_t w[kRowDw / 4];
#pragma unroll
      for (int i = 0; i < kRowDw / 4; ++i) w[i] = 0u;
      if (!k_unsafe) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int c = cq * 16 + e;
          w[e / kPer] |= quant_code_fast(x[e], gs[gi][c], gy[gi][c], gz[gi][c], BITS) << ((e % kPer) * BITS);
        }
      } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int c = cq * 16 + e;
          w[e / kPer] |= quant_code(x[e], gs[gi][c], gz[gi][c], BITS) << ((e % kPer) * BITS);
        }
      }
      uint32_t* out = reinterpret_cast<uint32_t*>(dst.kc) + ((size_t)h * Tcap + (size_t)u * kTile + r) * kRowDw + cq * (kRowDw / 4);
#pragma unroll
      for (int i = 0; i < kRowDw / 4; ++i) {
        out[i] = w[i];
        if (candidate) changed |= w[i] ^ k_in[i];
      }
    }
  } else if (row_valid) {
    uint4* out = reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(dst.kc) + ((size_t)h * Tcap + (size_t)u * kTile + r) * kD + cq * 16);
    uint32_t w[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) w[e] = (uint32_t)bf16_bits(x[2 * e]) | ((uint32_t)bf16_bits(x[2 * e + 1]) << 16);
    out[0] = make_uint4(w[0], w[1], w[2], w[3]);
    out[1] = make_uint4(w[4], w[5], w[6], w[7]);
  }

  // ---------------- values ----------------
  // "quantize once" (carry_values): a row that comes from the cache keeps its codes and parameters; a wave whose rows
  // all do skips the arithmetic altogether
  const bool carry = kQuant && CARRY && from_cache;
  const bool all_carried = kQuant && CARRY && __all(from_cache || !row_valid);
#pragma unroll
  for (int e = 0; e < 16; ++e) x[e] = 0.f;
  if (from_cache && !all_carried) {
    if constexpr (kQuant) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const uint32_t code = (vraw[e] >> v_shift) & kMask;
        x[e] = round_bf16(((float)code - v_pz) * v_ps);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e) x[e] = __uint_as_float(vraw[e] << 16);
    }
  } else if (row_valid) {
#pragma unroll
    for (int e = 0; e < 8; ++e) { x[2 * e] = bf16_lo(vraw[e]); x[2 * e + 1] = bf16_hi(vraw[e]); }
  }

  if constexpr (kQuant) {
    uint32_t vcode[16];
    QParam q;
    q.s = v_ps; q.z = v_pz; q.y = 0.f; q.safe = true;
    if (!all_carried) {  // (wave-uniform: the lane exchanges below are taken by whole waves)
      float lo = x[0], hi = x[0];
#pragma unroll
      for (int e = 1; e < 16; ++e) { lo = fminf(lo, x[e]); hi = fmaxf(hi, x[e]); }
      // the G channels of a group sit in G/16 neighbouring threads of the same token
      lo = fminf(lo, __shfl_xor(lo, 1));
      hi = fmaxf(hi, __shfl_xor(hi, 1));
      if (G == 64) {
        lo = fminf(lo, __shfl_xor(lo, 2));
        hi = fmaxf(hi, __shfl_xor(hi, 2));
      }
      q = group_param(lo, hi, BITS);
      if (__all(q.safe)) {
#pragma unroll
        for (int e = 0; e < 16; ++e) vcode[e] = quant_code_fast(x[e], q.s, q.y, q.z, BITS);
      } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) vcode[e] = quant_code(x[e], q.s, q.z, BITS);
      }
    }
    if (carry) {  // the row's own codes and parameters, as read
      q.s = v_ps;
      q.z = v_pz;
#pragma unroll
      for (int e = 0; e < 16; ++e) vcode[e] = (vraw[e] >> v_shift) & kMask;
    }
    if (row_valid && (cq * 16) % G == 0) {
      const size_t gidx = ((size_t)h * Tcap + (size_t)u * kTile + r) * kVGroups + (cq * 16) / G;
      dst.vs[gidx] = q.s;
      dst.vz[gidx] = q.z;
    }
    if (candidate && row_valid) changed |= (__float_as_uint(v_ps) ^ __float_as_uint(q.s)) | (__float_as_uint(v_pz) ^ __float_as_uint(q.z));
#pragma unroll
    for (int e = 0; e < 16; ++e) vt[cq * 16 + e][r] = row_valid ? (uint16_t)vcode[e] : (uint16_t)0;
    if (candidate && row_valid) {
#pragma unroll
      for (int e = 0; e < 16; ++e) changed |= vcode[e] ^ ((vraw[e] >> v_shift) & kMask);
    }
  } else {
#pragma unroll
    for (int e = 0; e < 16; ++e) vt[cq * 16 + e][r] = row_valid ? bf16_bits(x[e]) : (uint16_t)0;
  }
  __syncthreads();
  {  // thread = (channel tid/4, token quarter tid%4): 16 tokens of one channel → packed, coalesced
    const int c = tid >> 2, tq = tid & 3;
    const uint4 a0 = *reinterpret_cast<const uint4*>(&vt[c][tq * 16]);
    const uint4 a1 = *reinterpret_cast<const uint4*>(&vt[c][tq * 16 + 8]);
    const uint32_t ww[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
    if constexpr (kQuant) {
      uint32_t w[kRowDw / 4];
#pragma unroll
      for (int i = 0; i < kRowDw / 4; ++i) w[i] = 0u;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const uint32_t code = (e & 1) ? (ww[e >> 1] >> 16) : (ww[e >> 1] & 0xffffu);
        w[e / kPer] |= code << ((e % kPer) * BITS);
      }
      uint32_t* out = reinterpret_cast<uint32_t*>(dst.vc) + ((size_t)h * Tcap + (size_t)u * kTile + c) * kRowDw + tq * (kRowDw / 4);
#pragma unroll
      for (int i = 0; i < kRowDw / 4; ++i) out[i] = w[i];
    } else {
      uint4* out = reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(dst.vc) + ((size_t)h * Tcap + (size_t)u * kTile + c) * kD + tq * 16);
      out[0] = a0;
      out[1] = a1;
    }
  }
  if (candidate) {  // did the block reproduce itself?  (bf16 rows always do: they are copied)
    const int any = __syncthreads_or(changed != 0);
    if (tid == 0) *stable = any ? 0 : 1;
  } else if (tid == 0) {
    *stable = 0;  // a block whose rows may move carries no flag into a later step in which they do not
  }
}

// Clears the block flags (a kernel rather than a memset node: a caller may capture the stream, and memset nodes in
// captured graphs have replayed wrongly on this platform).
__global__ __launch_bounds__(256) void zero_bytes_kernel(uint8_t* p, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0;
}

hipError_t launch_zero_bytes(uint8_t* p, size_t n, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(zero_bytes_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p, n);
  return hipGetLastError();
}

hipError_t launch_requant(const RequantArgs& a, hipStream_t stream) {
  if (a.Tn <= 0) return hipSuccess;
  const dim3 grid((a.Tn + kTile - 1) / kTile, a.pool.H, a.b.n_layers);
  const int bits = a.pool.bits, G = a.pool.G;
  const bool carry = a.carry_values != 0 && bits != 16;
  if (bits == 16) hipLaunchKernelGGL((requant_kernel<16, 64>), grid, dim3(256), 0, stream, a);
  else if (bits == 4 && G == 64 && !carry) hipLaunchKernelGGL((requant_kernel<4, 64>), grid, dim3(256), 0, stream, a);
  else if (bits == 4 && G == 32 && !carry) hipLaunchKernelGGL((requant_kernel<4, 32>), grid, dim3(256), 0, stream, a);
  else if (bits == 2 && G == 64 && !carry) hipLaunchKernelGGL((requant_kernel<2, 64>), grid, dim3(256), 0, stream, a);
  else if (bits == 2 && G == 32 && !carry) hipLaunchKernelGGL((requant_kernel<2, 32>), grid, dim3(256), 0, stream, a);
  else if (bits == 4 && G == 64) hipLaunchKernelGGL((requant_kernel<4, 64, true>), grid, dim3(256), 0, stream, a);
  else if (bits == 4 && G == 32) hipLaunchKernelGGL((requant_kernel<4, 32, true>), grid, dim3(256), 0, stream, a);
  else if (bits == 2 && G == 64) hipLaunchKernelGGL((requant_kernel<2, 64, true>), grid, dim3(256), 0, stream, a);
  else if (bits == 2 && G == 32) hipLaunchKernelGGL((requant_kernel<2, 32, true>), grid, dim3(256), 0, stream, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

// ---- canonical unpack: thread per (head, token, channel) -------------------------------------------
template <int BITS>
__global__ __launch_bounds__(256) void unpack_kernel(const UnpackArgs a) {
  constexpr bool kQuant = BITS != 16;
  constexpr int kRowDw = kD * BITS / 32;
  constexpr int kPer = kQuant ? 32 / BITS : 2;
  constexpr uint32_t kMask = kQuant ? (1u << (BITS & 15)) - 1u : 0xffffu;
  const int H = a.pool.H, T = a.T, Tcap = a.pool.Tcap, G = a.pool.G;
  const size_t gid = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (gid >= (size_t)H * T * kD) return;
  const int c = (int)(gid % kD);
  const int t = (int)((gid / kD) % T);
  const int h = (int)(gid / ((size_t)kD * T));
  const LayerCache lc = layer_cache(a.pool, a.buf, a.layer);
  const uint32_t* krow = reinterpret_cast<const uint32_t*>(lc.kc) + ((size_t)h * Tcap + t) * kRowDw;
  const uint32_t* vrow = reinterpret_cast<const uint32_t*>(lc.vc) + ((size_t)h * Tcap + (size_t)(t / kTile) * kTile + c) * kRowDw;
  const uint32_t kcode = (krow[c / kPer] >> ((c % kPer) * BITS)) & kMask;
  const int col = t % kTile;
  const uint32_t vcode = (vrow[col / kPer] >> ((col % kPer) * BITS)) & kMask;
  if constexpr (kQuant) {
    const int ng = (T + G - 1) / G, vg = kD / G;
    const float ks = lc.ks[((size_t)h * (Tcap / G) + t / G) * kD + c], kz = lc.kz[((size_t)h * (Tcap / G) + t / G) * kD + c];
    const float vs = lc.vs[((size_t)h * Tcap + t) * vg + c / G], vz = lc.vz[((size_t)h * Tcap + t) * vg + c / G];
    if (a.k_codes) a.k_codes[gid] = (uint8_t)kcode;
    if (a.v_codes) a.v_codes[gid] = (uint8_t)vcode;
    if (t % G == 0) {
      if (a.k_scale) a.k_scale[((size_t)h * ng + t / G) * kD + c] = ks;
      if (a.k_zero) a.k_zero[((size_t)h * ng + t / G) * kD + c] = kz;
    }
    if (c % G == 0) {
      if (a.v_scale) a.v_scale[((size_t)h * T + t) * vg + c / G] = vs;
      if (a.v_zero) a.v_zero[((size_t)h * T + t) * vg + c / G] = vz;
    }
    if (a.k_bf16) a.k_bf16[gid] = bf16_bits(((float)kcode - kz) * ks);
    if (a.v_bf16) a.v_bf16[gid] = bf16_bits(((float)vcode - vz) * vs);
  } else {
    if (a.k_bf16) a.k_bf16[gid] = (uint16_t)kcode;
    if (a.v_bf16) a.v_bf16[gid] = (uint16_t)vcode;
  }
}

hipError_t launch_unpack(const UnpackArgs& a, hipStream_t stream) {
  const size_t total = (size_t)a.pool.H * a.T * kD;
  if (total == 0) return hipSuccess;
  const dim3 grid((unsigned)((total + 255) / 256));
  if (a.pool.bits == 16) hipLaunchKernelGGL((unpack_kernel<16>), grid, dim3(256), 0, stream, a);
  else if (a.pool.bits == 4) hipLaunchKernelGGL((unpack_kernel<4>), grid, dim3(256), 0, stream, a);
  else if (a.pool.bits == 2) hipLaunchKernelGGL((unpack_kernel<2>), grid, dim3(256), 0, stream, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace xsv
