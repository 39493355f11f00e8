// Token importance and keep-list selection (paper Sec. 3.2) for gfx950.
//
// The importance  S_j = (1/N_pooled) sum_i (Qbar Kbar^T)[i][j]  is linear in the pooled queries, so
// it is evaluated as  S_j = qtilde . Kbar_j  with  qtilde = (1/N_pooled) sum_i Qbar_i :
//   pool_query_kernel   one pass over Q: weighted row sums (weight 1/(H N_pooled) for a special
//                       row, 1/(H N_pooled |group|) for a patch row), kPoolSeg workgroups (row segments)
//                       and partials per head; every score workgroup adds the partials in a fixed
//                       order, so the result is reproducible bit for bit and needs no atomics.
//   score_kernel        one pass over the packed keys of the prunable middle: dequantized view,
//                       head mean, dot product with qtilde.  64 tokens x all heads per workgroup,
//                       16 channels per thread, all loads of a workgroup issued before any use.
//   Per-head variant (ScoreArgs::per_head, not the paper's): the averages over heads are left out,
//   qtilde_h comes from head h's partial alone and head h's keys give head h's own score vector.
//   select_kernel       exact top-k by radix select on order-preserving integer keys held in
//                       registers (4 passes of 8 bits, histograms in LDS, bin search by a shuffle
//                       scan), ties at the threshold resolved toward smaller positions, then an
//                       ordered compaction that emits the keep list ascending.
// Compiled with -ffp-contract=off: the dequantized view must be (code - zero) * scale with one
// rounding per operation.
#include "xsv_internal.h"

namespace xsv {

__device__ __forceinline__ float round_bf16(float x) { return (float)(__bf16)x; }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

constexpr int kPoolThreads = 1024;

// grid (H * kPoolSeg, layers), 1024 threads: thread = (row lane tid/8 of 128, channel run tid%8); a workgroup
// takes one of kPoolSeg row segments of one head.  One partial weighted row sum [64] per (head, segment);
// the score kernel adds the partials in (head, segment) order.
__global__ __launch_bounds__(kPoolThreads) void pool_query_kernel(const ScoreArgs a) {
  __shared__ float red[kPoolThreads / 8][kD + 1];
  const int lb = blockIdx.y, h = blockIdx.x / kPoolSeg, seg = blockIdx.x % kPoolSeg;
  const int H = a.pool.H, n = a.n, n_s = a.n_special, g = a.pool_size;
  const int seg_rows = (n + kPoolSeg - 1) / kPoolSeg, r_end = min(n, (seg + 1) * seg_rows);
  const int n_pooled = n_s + (n - n_s + g - 1) / g;
  const int tid = threadIdx.x, rl = tid >> 3, o = tid & 7;
  const uint16_t* qh = a.b.q[lb] + (size_t)h * a.b.q_sh;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const float base = a.per_head ? (float)n_pooled : (float)(H * n_pooled);
#pragma unroll 4
  for (int r = seg * seg_rows + rl; r < r_end; r += kPoolThreads / 8) {
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
  // fold the 128 row lanes in a fixed order: 4 segments of 32, then a chain
  __shared__ float seg4[4][kD];
  if (tid < 4 * kD) {
    const int sg = tid >> 6, c = tid & 63;
    float s = 0.f;
    for (int i = sg * 32; i < sg * 32 + 32; ++i) s += red[i][c];
    seg4[sg][c] = s;
  }
  __syncthreads();
  if (tid < kD) {
    float* part = a.ws.qpart + (size_t)(a.b.layer0 + lb) * a.ws.qpart_rows * kD;
    part[(size_t)blockIdx.x * kD + tid] = ((seg4[0][tid] + seg4[1][tid]) + seg4[2][tid]) + seg4[3][tid];
  }
}

hipError_t launch_pool_query(const ScoreArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(pool_query_kernel, dim3(a.pool.H * kPoolSeg, a.b.n_layers), dim3(kPoolThreads), 0, stream, a);
  return hipGetLastError();
}

// grid (blocks of 64 cache positions covering the middle, layers), 256 threads:
// thread = (token tid/4 of the block, channel quarter tid%4 = 16 channels).
// Everything a workgroup needs is requested up front (one memory round trip): the H partial query
// sums, the group parameters of all heads (staged in LDS, they are shared by the block's tokens)
// and the thread's packed codes of all heads.
template <int BITS, int G, int HMAX, bool PER_HEAD>
__global__ __launch_bounds__(256) void score_kernel(const ScoreArgs a) {
  constexpr bool kQuant = BITS != 16;
  constexpr int kGroups = kQuant ? kTile / G : 1;  // key groups inside a block of 64 positions
  constexpr int kRowDw = kD * BITS / 32;           // dwords per key row
  constexpr int kDwT = kRowDw / 4;                 // dwords per thread (16 channels)
  __shared__ float qtilde[PER_HEAD ? HMAX * kD : kD];  // per head: one row per head of the chunk
  __shared__ float prm[kQuant ? HMAX * kGroups * 2 * kD : 1];  // [head][group][scale|zero][channel]

  const int lb = blockIdx.y;
  const int H = a.pool.H;
  const int tid = threadIdx.x, r = tid >> 2, cq = tid & 3;
  const int block = a.T_first / kTile + blockIdx.x;
  const int pos = block * kTile + r;  // cache position
  const bool valid = pos >= a.T_first && pos < a.T_first + a.P;
  const bool plain = a.k_plain != nullptr;

  const uint32_t* src;
  size_t head_stride;  // dwords
  if (plain) {
    src = reinterpret_cast<const uint32_t*>(a.k_plain) + (size_t)(pos - a.T_first) * kRowDw + cq * kDwT;
    head_stride = (size_t)a.P * kRowDw;
  } else {
    const LayerCache lc = layer_cache(a.pool, a.b.src_buf(lb), a.b.layer0 + lb);
    src = reinterpret_cast<const uint32_t*>(lc.kc) + (size_t)pos * kRowDw + cq * kDwT;
    head_stride = (size_t)a.pool.Tcap * kRowDw;
  }
  const float* part = a.ws.qpart + (size_t)(a.b.layer0 + lb) * a.ws.qpart_rows * kD;

  auto fold_partials = [&]() {  // the H partial query sums, in head order (called once, behind the chunk's loads)
    if (!PER_HEAD && tid < kD) {
      float s = 0.f;
#pragma unroll 16
      for (int h = 0; h < H * kPoolSeg; ++h) s += part[(size_t)h * kD + tid];
      qtilde[tid] = s;
    }
  };
  float acc[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  for (int h0 = 0; h0 < H; h0 += HMAX) {  // heads in chunks of HMAX (one chunk for H <= HMAX)
    const int hn = min(HMAX, H - h0);
    // codes (or bf16 rows) of this thread's 16 channels, all heads of the chunk
    uint32_t w[HMAX][kDwT];
#pragma unroll
    for (int h = 0; h < HMAX; ++h)
#pragma unroll
      for (int i = 0; i < kDwT; ++i) w[h][i] = (valid && h < hn) ? src[(h0 + h) * head_stride + i] : 0u;
    if constexpr (PER_HEAD) {
      if (h0 > 0) __syncthreads();  // the previous chunk's rows are no longer read
      for (int i = tid; i < hn * kD; i += 256) {  // head h0 + i / 64: its segments in order
        const float* ph = part + ((size_t)(h0 + i / kD) * kPoolSeg) * kD + i % kD;
        float s = ph[0];
#pragma unroll
        for (int sg = 1; sg < kPoolSeg; ++sg) s += ph[sg * kD];
        qtilde[i] = s;
      }
    }
    if constexpr (kQuant) {
      const LayerCache lc = layer_cache(a.pool, a.b.src_buf(lb), a.b.layer0 + lb);
      const int gcap = a.pool.Tcap / G;
      constexpr int kPrmIter = HMAX * kGroups * 2 * kD / 256;
      float pr[kPrmIter];  // loaded first, stored to LDS below: every load is in flight before the first wait
#pragma unroll
      for (int it = 0; it < kPrmIter; ++it) {
        const int i = tid + it * 256;
        const int c = i % kD, sz = (i / kD) & 1, gi = (i / (2 * kD)) % kGroups, h = i / (2 * kD * kGroups);
        const float* p = sz ? lc.kz : lc.ks;
        pr[it] = h < hn ? p[((size_t)(h0 + h) * gcap + block * kGroups + gi) * kD + c] : 0.f;
      }
      if (h0 == 0) fold_partials();
      if (h0 > 0 && !PER_HEAD) __syncthreads();  // the previous chunk's parameters are no longer read
#pragma unroll
      for (int it = 0; it < kPrmIter; ++it) prm[tid + it * 256] = pr[it];
    } else {
      if (h0 == 0) fold_partials();
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < HMAX; ++h) {
      if (h < hn) {
        float x[16];  // head h's key row (this thread's 16 channels), dequantized view
        if constexpr (kQuant) {
          const float* ks = prm + ((h * kGroups + (r / G) % kGroups) * 2) * kD + cq * 16;
          const float* kz = ks + kD;
          // codes to floats by bytes: one mask per 4 (4-bit: per 8) codes, then one byte-to-float conversion each,
          // instead of a bit-field extract and a conversion per code
          float code[16];
#pragma unroll
          for (int d = 0; d < kDwT; ++d) {
            constexpr int kPerDw = 32 / BITS;  // 8 or 16 codes per dword
#pragma unroll
            for (int sft = 0; sft < 8 / BITS; ++sft) {  // code e of the dword sits in byte e / (8 / BITS) of (w >> BITS * (e % (8 / BITS))) & mask
              uint32_t t = (w[h][d] >> (BITS * sft)) & (BITS == 4 ? 0x0f0f0f0fu : 0x03030303u);
              asm volatile("" : "+v"(t));  // (keeps the mask shared by the four conversions below)
#pragma unroll
              for (int b = 0; b < 4; ++b) code[d * kPerDw + b * (8 / BITS) + sft] = (float)((t >> (8 * b)) & 0xffu);
            }
          }
          // canonical view, rounded to bf16 in pairs (one packed conversion per two values)
#pragma unroll
          for (int e = 0; e < 16; e += 2) {
            typedef __attribute__((ext_vector_type(2))) float f2;
            typedef __attribute__((ext_vector_type(2))) __bf16 b2;
            const f2 v = {(code[e] - kz[e]) * ks[e], (code[e + 1] - kz[e + 1]) * ks[e + 1]};
            const uint32_t pk = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, b2));
            x[e] = bf16_lo(pk);
            x[e + 1] = bf16_hi(pk);
          }
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            x[2 * e] = bf16_lo(w[h][e]);
            x[2 * e + 1] = bf16_hi(w[h][e]);
          }
        }
        if constexpr (PER_HEAD) {
          const float* qt = qtilde + h * kD + cq * 16;
          float dot = 0.f;
#pragma unroll
          for (int e = 0; e < 16; ++e) dot += qt[e] * x[e];
          dot += __shfl_xor(dot, 1);
          dot += __shfl_xor(dot, 2);
          if (valid && cq == 0)
            a.ws.scores[list_index(a.ws.sets, a.b.layer0 + lb, h0 + h) * a.ws.scores_stride + (pos - a.T_first)] = dot;
        } else {
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[e] += x[e];
        }
      }
    }
  }
  if constexpr (PER_HEAD) return;
  const float* qt = qtilde + cq * 16;
  float dot = 0.f;
  const float fH = (float)H;
#pragma unroll
  for (int e = 0; e < 16; ++e) dot += qt[e] * (acc[e] / fH);
  dot += __shfl_xor(dot, 1);
  dot += __shfl_xor(dot, 2);
  if (valid && cq == 0) a.ws.scores[list_index(a.ws.sets, a.b.layer0 + lb, 0) * a.ws.scores_stride + (pos - a.T_first)] = dot;
}

template <bool PER_HEAD>
static hipError_t launch_score_t(const ScoreArgs& a, hipStream_t stream) {
  const int first_block = a.T_first / kTile;
  const int last_block = (a.T_first + a.P - 1) / kTile;
  const dim3 grid(last_block - first_block + 1, a.b.n_layers);
  const int bits = a.k_plain ? 16 : a.pool.bits, G = a.pool.G;
  if (bits == 16) hipLaunchKernelGGL((score_kernel<16, 64, 16, PER_HEAD>), grid, dim3(256), 0, stream, a);
  else if (bits == 4 && G == 64) hipLaunchKernelGGL((score_kernel<4, 64, 16, PER_HEAD>), grid, dim3(256), 0, stream, a);
  else if (bits == 4 && G == 32) hipLaunchKernelGGL((score_kernel<4, 32, 16, PER_HEAD>), grid, dim3(256), 0, stream, a);
  else if (bits == 2 && G == 64) hipLaunchKernelGGL((score_kernel<2, 64, 16, PER_HEAD>), grid, dim3(256), 0, stream, a);
  else if (bits == 2 && G == 32) hipLaunchKernelGGL((score_kernel<2, 32, 16, PER_HEAD>), grid, dim3(256), 0, stream, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_score(const ScoreArgs& a, hipStream_t stream) {
  return a.per_head ? launch_score_t<true>(a, stream) : launch_score_t<false>(a, stream);
}

// ---- selection --------------------------------------------------------------------------------------

// float → unsigned key with the same order (larger score ↔ larger key); -0 and +0 stay distinct
// neighbours, which only matters for exact-zero scores.
__device__ __forceinline__ uint32_t order_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int kSelThreads = 256;  // 4 waves: cheap barriers; one histogram bin per thread

// exclusive prefix sums of two counters over the workgroup's threads, in thread order
__device__ __forceinline__ void block_exclusive_scan2(int& a, int& b, int* sh /* 2*16 */, int& total_a, int& total_b) {
  static_assert(kSelThreads / 64 <= 16, "wave totals live in 16 slots");
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

// one workgroup per list (layer, or layer and head); KPT > 0: each thread keeps its (at most KPT) keys in registers
template <int KPT>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const SelectArgs a) {
  __shared__ int hist[256];
  __shared__ int wave_tot[4];
  __shared__ int sh_scan[32];
  __shared__ uint32_t sh_prefix;
  __shared__ int sh_need;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* scores = a.scores + (size_t)blockIdx.x * a.scores_stride;
  int32_t* keep = a.keep + (size_t)blockIdx.x * a.keep_stride;
  const int P = a.P, k = a.k;

  // thread t owns the contiguous positions [t*per, (t+1)*per)
  const int per = (P + kSelThreads - 1) / kSelThreads;
  const int j0 = min(P, tid * per), j1 = min(P, j0 + per);
  uint32_t keys[KPT > 0 ? KPT : 1];
  if constexpr (KPT > 0) {
#pragma unroll
    for (int i = 0; i < KPT; ++i) keys[i] = (j0 + i < j1) ? order_key(scores[j0 + i]) : 0u;
  }
  auto key_at = [&](int i) -> uint32_t {  // i-th key of this thread
    if constexpr (KPT > 0) return keys[i];
    else return order_key(scores[j0 + i]);
  };

  // k-th largest key by radix select, most significant byte first
  uint32_t prefix = 0;
  int need = k;  // rank still to find inside the current prefix class (1-based from the top)
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    hist[tid] = 0;
    __syncthreads();
    const uint32_t hi_mask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
    if constexpr (KPT > 0) {
#pragma unroll
      for (int i = 0; i < KPT; ++i)
        if (j0 + i < j1 && (keys[i] & hi_mask) == prefix) atomicAdd(&hist[(keys[i] >> shift) & 255u], 1);
    } else {
      for (int i = 0; i < j1 - j0; ++i) {
        const uint32_t key = key_at(i);
        if ((key & hi_mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
      }
    }
    __syncthreads();
    // bin b holds the wanted rank iff  (#keys in bins above b) < need <= (that + hist[b]);
    // suffix sums over the 256 bins: per-wave shuffle scan + 4 wave totals
    const int h = hist[tid];
    int incl = h;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int v = __shfl_down(incl, d);
      if (lane + d < 64) incl += v;
    }
    if (lane == 0) wave_tot[wave] = incl;
    __syncthreads();
    int above = incl - h;
    for (int w = wave + 1; w < 4; ++w) above += wave_tot[w];
    if (above < need && need <= above + h) {
      sh_prefix = prefix | ((uint32_t)tid << shift);
      sh_need = need - above;
    }
    __syncthreads();
    prefix = sh_prefix;
    need = sh_need;
  }
  const uint32_t thr = prefix;  // key of the k-th largest score
  const int need_eq = need;     // how many of the scores equal to it are kept (smallest positions)

  // ordered compaction
  int n_gt = 0, n_eq = 0;
  for (int i = 0; i < j1 - j0; ++i) {
    const uint32_t key = key_at(i);
    n_gt += key > thr;
    n_eq += key == thr;
  }
  int gt_before = n_gt, eq_before = n_eq, tot_gt, tot_eq;
  block_exclusive_scan2(gt_before, eq_before, sh_scan, tot_gt, tot_eq);
  int out = a.T_first + gt_before + min(eq_before, need_eq);
  int eq_rank = eq_before;
  for (int i = 0; i < j1 - j0; ++i) {
    const uint32_t key = key_at(i);
    bool take = key > thr;
    if (key == thr) {
      take = eq_rank < need_eq;
      ++eq_rank;
    }
    if (take) keep[out++] = a.T_first + j0 + i;
  }
  for (int i = tid; i < a.T_first; i += kSelThreads) keep[i] = i;
  for (int i = tid; i < a.T_cur; i += kSelThreads) keep[a.T_first + k + i] = a.T_first + P + i;
}

hipError_t launch_select(const SelectArgs& a, hipStream_t stream) {
  static_assert(kSelThreads == 256, "one histogram bin per thread");
  if (a.P <= 16 * kSelThreads) hipLaunchKernelGGL(select_kernel<16>, dim3(a.n_lists), dim3(kSelThreads), 0, stream, a);
  else if (a.P <= 32 * kSelThreads) hipLaunchKernelGGL(select_kernel<32>, dim3(a.n_lists), dim3(kSelThreads), 0, stream, a);
  else hipLaunchKernelGGL(select_kernel<0>, dim3(a.n_lists), dim3(kSelThreads), 0, stream, a);
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

hipError_t launch_fill_keep(int32_t* keep, int keep_stride, int n_lists, int T_first, int P, int T_cur, bool keep_middle,
                            hipStream_t stream) {
  const int total = T_first + (keep_middle ? P : 0) + T_cur;
  if (total <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_keep_kernel, dim3((total + 255) / 256, n_lists), dim3(256), 0, stream, keep, keep_stride,
                     T_first, P, T_cur, keep_middle ? 1 : 0);
  return hipGetLastError();
}

}  // namespace xsv
