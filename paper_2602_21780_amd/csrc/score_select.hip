// Token importance and keep-list selection (paper Sec. 3.2) for gfx950.
//
// The importance  S_j = (1/N_pooled) sum_i (Qbar Kbar^T)[i][j]  is linear in the pooled queries, so
// it is evaluated as  S_j = qtilde . Kbar_j  with  qtilde = (1/N_pooled) sum_i Qbar_i :
//   pool_query_kernel   one pass over Q: weighted row sums (weight 1/(H N_pooled) for a special
//                       row, 1/(H N_pooled |group|) for a patch row) per workgroup; the partials are
//                       folded in a fixed order by every score workgroup, so the result is
//                       reproducible bit for bit and needs no atomics.
//   score_kernel        one pass over the packed keys of the prunable middle: dequantized view,
//                       head mean, dot product with qtilde.  HBM-bound: 64 tokens x all heads per
//                       workgroup, 16 channels per thread, coalesced 8-byte code loads.
//   select_kernel       exact top-k by radix select on order-preserving integer keys (4 passes of
//                       8 bits, histograms in LDS), ties at the threshold resolved toward smaller
//                       positions, then an ordered compaction that emits the keep list ascending.
// Compiled with -ffp-contract=off: the dequantized view must be (code - zero) * scale with one
// rounding per operation.
#include "xsv_internal.h"

namespace xsv {

__device__ __forceinline__ float round_bf16(float x) { return (float)(__bf16)x; }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

constexpr int kPoolRows = 128;  // query rows per workgroup of pool_query_kernel

// grid (chunks, H, layers), 256 threads: thread = (row lane tid/8 of 32, channel run tid%8)
__global__ __launch_bounds__(256) void pool_query_kernel(const ScoreArgs a) {
  __shared__ float red[32][kD + 1];
  const int lb = blockIdx.z, h = blockIdx.y, chunk = blockIdx.x;
  const int H = a.pool.H, n = a.n, n_s = a.n_special, g = a.pool_size;
  const int n_pooled = n_s + (n - n_s + g - 1) / g;
  const int tid = threadIdx.x, rl = tid >> 3, o = tid & 7;
  const uint16_t* qh = a.b.q[lb] + (size_t)h * a.b.q_sh;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const float base = (float)(H * n_pooled);
  for (int r = chunk * kPoolRows + rl; r < min(n, (chunk + 1) * kPoolRows); r += 32) {
    float w;
    if (r < n_s) {
      w = 1.0f / base;
    } else {
      const int u = (r - n_s) / g;
      const int size = min(g, n - n_s - u * g);
      w = 1.0f / (base * (float)size);
    }
    const uint4 v = *reinterpret_cast<const uint4*>(qh + (size_t)r * a.b.q_st + o * 8);
    const uint32_t ww[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      acc[2 * e] += w * bf16_lo(ww[e]);
      acc[2 * e + 1] += w * bf16_hi(ww[e]);
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) red[rl][o * 8 + e] = acc[e];
  __syncthreads();
  float* part = a.ws.qpart + (size_t)(a.b.layer0 + lb) * a.ws.qpart_rows * kD;
  if (tid < kD) {
    float s = 0.f;
    for (int i = 0; i < 32; ++i) s += red[i][tid];
    part[(size_t)(h * gridDim.x + chunk) * kD + tid] = s;
  }
}

hipError_t launch_pool_query(const ScoreArgs& a, hipStream_t stream) {
  const int chunks = (a.n + kPoolRows - 1) / kPoolRows;
  hipLaunchKernelGGL(pool_query_kernel, dim3(chunks, a.pool.H, a.b.n_layers), dim3(256), 0, stream, a);
  return hipGetLastError();
}

// grid (blocks of 64 cache positions covering the middle, layers), 256 threads:
// thread = (token tid/4 of the block, channel quarter tid%4 = 16 channels)
template <int BITS, int G>
__global__ __launch_bounds__(256) void score_kernel(const ScoreArgs a) {
  const int lb = blockIdx.y;
  const int H = a.pool.H;
  const int tid = threadIdx.x, r = tid >> 2, cq = tid & 3;
  const int first_block = a.T_first / kTile;
  const int pos = (first_block + blockIdx.x) * kTile + r;  // cache position
  const bool valid = pos >= a.T_first && pos < a.T_first + a.P;

  // qtilde: fold the per-workgroup partial query sums in a fixed order (4 segments, then a chain)
  __shared__ float seg[4][kD];
  __shared__ float qtilde[kD];
  {
    const int n_parts = ((a.n + kPoolRows - 1) / kPoolRows) * H;
    const float* part = a.ws.qpart + (size_t)(a.b.layer0 + lb) * a.ws.qpart_rows * kD;
    const int per = (n_parts + 3) / 4, sg = tid >> 6, c = tid & 63;
    float s = 0.f;
    for (int i = sg * per; i < min(n_parts, (sg + 1) * per); ++i) s += part[(size_t)i * kD + c];
    seg[sg][c] = s;
    __syncthreads();
    if (tid < kD) qtilde[tid] = ((seg[0][tid] + seg[1][tid]) + seg[2][tid]) + seg[3][tid];
    __syncthreads();
  }
  const float* qt = qtilde + cq * 16;

  float acc[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;

  if (valid) {
    if (a.k_plain != nullptr || BITS == 16) {
      // bf16 rows: the plain tensor [H][P][64] of the stateless form, or the bf16 cache
      const uint16_t* base;
      size_t head_stride;
      if (a.k_plain != nullptr) {
        base = a.k_plain + (size_t)(pos - a.T_first) * kD;
        head_stride = (size_t)a.P * kD;
      } else {
        const LayerCache lc = layer_cache(a.pool, a.b.src_buf(lb), a.b.layer0 + lb);
        base = reinterpret_cast<const uint16_t*>(lc.kc) + (size_t)pos * kD;
        head_stride = (size_t)a.pool.Tcap * kD;
      }
      for (int h = 0; h < H; ++h) {
        const uint4* p = reinterpret_cast<const uint4*>(base + h * head_stride + cq * 16);
        const uint4 v0 = p[0], v1 = p[1];
        const uint32_t ww[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          acc[2 * e] += bf16_lo(ww[e]);
          acc[2 * e + 1] += bf16_hi(ww[e]);
        }
      }
    } else {
      const LayerCache lc = layer_cache(a.pool, a.b.src_buf(lb), a.b.layer0 + lb);
      constexpr int kRowDw = kD * BITS / 32;   // dwords per key row
      constexpr int kDwPerThread = kRowDw / 4;  // 16 channels
      constexpr uint32_t mask = (1u << BITS) - 1u;
      const int gcap = a.pool.Tcap / G;
      for (int h = 0; h < H; ++h) {
        const uint32_t* codes = reinterpret_cast<const uint32_t*>(lc.kc) + ((size_t)h * a.pool.Tcap + pos) * kRowDw + cq * kDwPerThread;
        const float* ks = lc.ks + ((size_t)h * gcap + pos / G) * kD + cq * 16;
        const float* kz = lc.kz + ((size_t)h * gcap + pos / G) * kD + cq * 16;
        uint32_t w[kDwPerThread];
#pragma unroll
        for (int i = 0; i < kDwPerThread; ++i) w[i] = codes[i];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const uint32_t code = (w[(e * BITS) / 32] >> ((e * BITS) % 32)) & mask;
          acc[e] += round_bf16(((float)code - kz[e]) * ks[e]);
        }
      }
    }
  }
  float dot = 0.f;
  const float fH = (float)H;
#pragma unroll
  for (int e = 0; e < 16; ++e) dot += qt[e] * (acc[e] / fH);
  dot += __shfl_xor(dot, 1);
  dot += __shfl_xor(dot, 2);
  if (valid && cq == 0) a.ws.scores[(size_t)(a.b.layer0 + lb) * a.ws.scores_stride + (pos - a.T_first)] = dot;
}

hipError_t launch_score(const ScoreArgs& a, hipStream_t stream) {
  const int first_block = a.T_first / kTile;
  const int last_block = (a.T_first + a.P - 1) / kTile;
  const dim3 grid(last_block - first_block + 1, a.b.n_layers);
  const int bits = a.k_plain ? 16 : a.pool.bits, G = a.pool.G;
  if (bits == 16) hipLaunchKernelGGL((score_kernel<16, 64>), grid, dim3(256), 0, stream, a);
  else if (bits == 4 && G == 64) hipLaunchKernelGGL((score_kernel<4, 64>), grid, dim3(256), 0, stream, a);
  else if (bits == 4 && G == 32) hipLaunchKernelGGL((score_kernel<4, 32>), grid, dim3(256), 0, stream, a);
  else if (bits == 2 && G == 64) hipLaunchKernelGGL((score_kernel<2, 64>), grid, dim3(256), 0, stream, a);
  else if (bits == 2 && G == 32) hipLaunchKernelGGL((score_kernel<2, 32>), grid, dim3(256), 0, stream, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

// ---- selection --------------------------------------------------------------------------------------

// float → unsigned key with the same order (larger score ↔ larger key); -0 and +0 stay distinct
// neighbours, which only matters for exact-zero scores.
__device__ __forceinline__ uint32_t order_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int kSelThreads = 1024;

// exclusive prefix sums of two counters over the workgroup's threads, in thread order
__device__ __forceinline__ void block_exclusive_scan2(int& a, int& b, int* sh /* 2*16 */, int& total_a, int& total_b) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int ia = a, ib = b;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int ta = __shfl_up(ia, d), tb = __shfl_up(ib, d);
    if (lane >= d) { ia += ta; ib += tb; }
  }
  if (lane == 63) { sh[wave] = ia; sh[16 + wave] = ib; }
  __syncthreads();
  int oa = 0, ob = 0;
  total_a = 0; total_b = 0;
  for (int w = 0; w < kSelThreads / 64; ++w) {
    if (w < wave) { oa += sh[w]; ob += sh[16 + w]; }
    total_a += sh[w]; total_b += sh[16 + w];
  }
  a = oa + ia - a;
  b = ob + ib - b;
  __syncthreads();
}

// one workgroup per layer
__global__ __launch_bounds__(kSelThreads) void select_kernel(const SelectArgs a) {
  __shared__ int hist[256];
  __shared__ int sh_scan[32];
  __shared__ uint32_t sh_prefix;
  __shared__ int sh_need;
  const int tid = threadIdx.x;
  const float* scores = a.scores + (size_t)blockIdx.x * a.scores_stride;
  int32_t* keep = a.keep + (size_t)blockIdx.x * a.keep_stride;
  const int P = a.P, k = a.k;

  // k-th largest key by radix select, most significant byte first
  uint32_t prefix = 0;
  int need = k;  // rank still to find inside the current prefix class (1-based from the top)
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    const uint32_t hi_mask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
    for (int j = tid; j < P; j += kSelThreads) {
      const uint32_t key = order_key(scores[j]);
      if ((key & hi_mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
    }
    __syncthreads();
    if (tid == 0) {
      int cum = 0, bin = 255;
      for (; bin > 0; --bin) {
        if (cum + hist[bin] >= need) break;
        cum += hist[bin];
      }
      sh_prefix = prefix | ((uint32_t)bin << shift);
      sh_need = need - cum;
    }
    __syncthreads();
    prefix = sh_prefix;
    need = sh_need;
    __syncthreads();
  }
  const uint32_t thr = prefix;  // key of the k-th largest score
  const int need_eq = need;     // how many of the scores equal to it are kept (smallest positions)

  // ordered compaction: thread t owns the contiguous positions [t*per, (t+1)*per)
  const int per = (P + kSelThreads - 1) / kSelThreads;
  const int j0 = min(P, tid * per), j1 = min(P, j0 + per);
  int n_gt = 0, n_eq = 0;
  for (int j = j0; j < j1; ++j) {
    const uint32_t key = order_key(scores[j]);
    n_gt += key > thr;
    n_eq += key == thr;
  }
  int gt_before = n_gt, eq_before = n_eq, tot_gt, tot_eq;
  block_exclusive_scan2(gt_before, eq_before, sh_scan, tot_gt, tot_eq);
  int out = a.T_first + gt_before + min(eq_before, need_eq);
  int eq_rank = eq_before;
  for (int j = j0; j < j1; ++j) {
    const uint32_t key = order_key(scores[j]);
    bool take = key > thr;
    if (key == thr) {
      take = eq_rank < need_eq;
      ++eq_rank;
    }
    if (take) keep[out++] = a.T_first + j;
  }
  for (int i = tid; i < a.T_first; i += kSelThreads) keep[i] = i;
  for (int i = tid; i < a.T_cur; i += kSelThreads) keep[a.T_first + k + i] = a.T_first + P + i;
}

hipError_t launch_select(const SelectArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(select_kernel, dim3(a.n_layers), dim3(kSelThreads), 0, stream, a);
  return hipGetLastError();
}

// keep = [0, T_first) ∪ (middle, if kept) ∪ current
__global__ __launch_bounds__(256) void fill_keep_kernel(int32_t* keep, int keep_stride, int T_first, int P, int T_cur,
                                                        int keep_middle) {
  int32_t* out = keep + (size_t)blockIdx.y * keep_stride;
  const int total = T_first + (keep_middle ? P : 0) + T_cur;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  out[i] = (keep_middle || i < T_first) ? i : i + P;
}

hipError_t launch_fill_keep(int32_t* keep, int keep_stride, int n_layers, int T_first, int P, int T_cur, bool keep_middle,
                            hipStream_t stream) {
  const int total = T_first + (keep_middle ? P : 0) + T_cur;
  if (total <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_keep_kernel, dim3((total + 255) / 256, n_layers), dim3(256), 0, stream, keep, keep_stride,
                     T_first, P, T_cur, keep_middle ? 1 : 0);
  return hipGetLastError();
}

}  // namespace xsv
