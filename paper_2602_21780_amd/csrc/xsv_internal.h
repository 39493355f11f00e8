// Internal layouts shared by the host API and the HIP kernels of libxsv (not part of the ABI).
//
// Packed cache of one layer (per head), private to the library:
//   keys    kc  [Tcap][64*bits/8 B]     one row per token, channel c at bit c*bits (little endian)
//           ks, kz [Tcap/G][64] fp32    scale / zero point per (group of G tokens, channel)
//   values  vc  [Tcap/64][64][64*bits/8 B]  blocks of 64 tokens, TRANSPOSED: one row per channel,
//                                       token j of the block at bit j*bits — so that 8 (16) tokens
//                                       of one channel are one dword, the unit the PV MFMA consumes
//           vs, vz [Tcap][64/G] fp32    scale / zero point per (token, group of G channels)
//   bits == 16: kc rows are 64 bf16, vc rows are 64 bf16 (still transposed in 64-token blocks).
//   token ids   tok_frame, tok_index [sets][Tcap] per layer; sets = 1 (one retained index set per layer, shared by
//               the heads) or H (one per head, see xsv_config.score_mode)
// Every layer has two such buffers; a step reads one and writes the other.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace xsv {

constexpr int kD = 64;         // head_dim
constexpr int kTile = 64;      // tokens per value block and per attention key tile
constexpr int kMaxBatch = 32;  // layers per batched launch
// Row segments (workgroups) per head of the pooled-query pass.  One: beside the attention launch of a step
// only a few compute units are idle when the chain starts, and with four segments (3 us faster alone) the
// extra workgroups wait for units and the step as a whole gets 1.6 % slower.
constexpr int kPoolSeg = 1;

struct CachePool {
  uint8_t* kc;
  float* ks;
  float* kz;
  uint8_t* vc;
  float* vs;
  float* vz;
  int32_t* tok_frame;
  int32_t* tok_index;
  int L, H, Tcap, bits, G;
  int sets;  // retained index sets per layer: 1, or H when every head selects for itself
  int buffers;  // 2: a step reads one buffer and writes the other; 1 (a cache that is never pruned: rows never move):
                // a step rewrites the blocks it touches in place

  // slab = one (buffer, layer); sizes in elements of the respective array
  __host__ __device__ size_t code_row_bytes() const { return (size_t)kD * bits / 8; }
  __host__ __device__ size_t code_slab() const { return (size_t)H * Tcap * code_row_bytes(); }
  __host__ __device__ size_t kparam_slab() const { return (size_t)H * (Tcap / G) * kD; }
  __host__ __device__ size_t vparam_slab() const { return (size_t)H * Tcap * (kD / G); }
  __host__ __device__ size_t tok_slab() const { return (size_t)(sets > 1 ? sets : 1) * Tcap; }
  __host__ __device__ size_t slab_index(int buf, int layer) const { return (size_t)buf * L + layer; }
};

// index of the score vector / keep list / token-id row that head h of `layer` uses
__host__ __device__ inline size_t list_index(int sets, int layer, int h) {
  return sets > 1 ? (size_t)layer * sets + h : (size_t)layer;
}

// One layer's view of the pool (device pointers of one buffer), head 0.
struct LayerCache {
  uint8_t* kc;
  float* ks;
  float* kz;
  uint8_t* vc;
  float* vs;
  float* vz;
  int32_t* tok_frame;
  int32_t* tok_index;
};

__host__ __device__ inline LayerCache layer_cache(const CachePool& p, int buf, int layer) {
  const size_t i = p.slab_index(buf, layer);
  LayerCache c;
  c.kc = p.kc + i * p.code_slab();
  c.vc = p.vc + i * p.code_slab();
  c.ks = p.ks ? p.ks + i * p.kparam_slab() : nullptr;
  c.kz = p.kz ? p.kz + i * p.kparam_slab() : nullptr;
  c.vs = p.vs ? p.vs + i * p.vparam_slab() : nullptr;
  c.vz = p.vz ? p.vz + i * p.vparam_slab() : nullptr;
  c.tok_frame = p.tok_frame + i * p.tok_slab();
  c.tok_index = p.tok_index + i * p.tok_slab();
  return c;
}

// The layers one launch works on, and their frame tensors.
struct Batch {
  int n_layers;     // layers in this launch
  int layer0;       // pool index of the first
  uint32_t bufsel;  // bit i: buffer that currently holds layer (layer0+i)'s cache
  const uint16_t* q[kMaxBatch];
  const uint16_t* k[kMaxBatch];
  const uint16_t* v[kMaxBatch];
  uint16_t* out[kMaxBatch];
  int64_t q_sh, q_st, k_sh, k_st, v_sh, v_st;  // strides in elements

  __host__ __device__ int src_buf(int i) const { return (bufsel >> i) & 1; }
};

// Per-layer workspaces (device), indexed by pool layer.
struct Workspace {
  float* scores;      // [L][sets][Tcap + n]  importance of the middle tokens
  int32_t* keep;      // [L][sets][Tcap + n]  keep list
  float* qpart;       // [L][qpart_rows = H * kPoolSeg][64] partial weighted query sums
  uint16_t* attn_o;   // [pieces][batch layers][H][ceil(n/32)] blocks of 32 rows x 64 fp16 mantissas of the unnormalized
                      // partial outputs, each block stored [16-byte piece 0..3][lane half][row] (4 KB)
  float* attn_ml;     // [pieces][batch layers][H][n][4]  softmax reference (log2 domain), row sum, row scale, -
  int scores_stride;  // Tcap + n
  int qpart_rows;
  int sets;           // lists per layer (CachePool::sets)
};

// ---- launchers (defined in the .hip files; every one only enqueues on `stream`) -----------------

constexpr int kMaxPieces = 16;  // workgroups that may share one unit
// One layer of an attention launch: device pointers at head 0 of the buffer that holds the layer's cache, and of the
// frame's tensors.  (Resolved on the host: a workgroup's first tile waits behind whatever address arithmetic the
// kernel has to do, and the argument block stays small.)
struct AttendLayer {
  const uint32_t* kc;
  const float* ks;
  const float* kz;
  const uint32_t* vc;
  const float* vs;
  const float* vz;
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  uint16_t* out;
};
struct AttendArgs {
  AttendLayer layer[kMaxBatch];
  int n_layers, H, bits, G;
  int Tcap;
  uint32_t code_head, kparam_head, vparam_head;  // elements (dwords / floats) between two heads of kc|vc, ks|kz, vs|vz
  int64_t q_sh, q_st, k_sh, k_st, v_sh, v_st;    // strides of the frame tensors in elements
  uint16_t* attn_o;  // partial outputs of cut units, see Workspace
  float* attn_ml;
  int Tc, n;
  int variant;   // waves x query rows per wave of a workgroup: 0: 4 x 64, 1: 4 x 32, 2: 8 x 32, 3: 8 x 64
  int n_wgs;     // workgroups the (unit, tile) line is cut into (from plan_attend)
  int rows_wg;   // query rows per workgroup of this variant
  int cut;       // some unit is shared by several workgroups: partials are written and merged
  int equal_ranges;  // > 0: every unit is cut into exactly this many key ranges, at the same tiles:
  // range p of a unit is its tiles [range_begin[p], range_begin[p + 1]); chosen on the host so that the ranges
  // COST the same (a tile of the frame's own bf16 rows takes longer to stage than a tile of packed codes), or
  // so that the last one is deliberately short (see xsv_set_short_range)
  int32_t range_begin[17];
  int xcd_ranges;  // > 0: every unit is cut into this many key ranges and the grid is permuted for L2 sharing
  float qscale;  // softmax scale * log2(e)
};
struct AttendPlan {
  int n_wgs, rows_wg, max_pieces;
};
// Chooses the grid: at most want_wgs workgroups, pieces of at least 4 tiles, and no unit shared by
// more workgroups than the partial workspace (part_rows rows) and the merge can hold.
AttendPlan plan_attend(int variant, int n_layers, int H, int n, int Tc, int want_wgs, size_t part_rows);
void partition_query(long long n_units, int n_tiles, int n_wgs, int wg, long long* begin, long long* end);
void partition_unit_query(long long n_units, int n_tiles, int n_wgs, int unit, int* first_wg, int* last_wg);
// `between` (optional): an event recorded after the attention kernel, before the merge kernel.
hipError_t launch_attend(const AttendArgs& a, hipStream_t stream, hipEvent_t between = nullptr);
int attend_rows_per_workgroup(int variant);

struct ScoreArgs {
  CachePool pool;
  Batch b;
  Workspace ws;
  int Tc, n, n_special, pool_size;
  int T_first, P;  // middle = cache positions [T_first, T_first + P)
  // stateless form: keys come from a plain bf16 tensor [H][P][64] instead of the pool
  const uint16_t* k_plain;
  int per_head;  // 1: no averages over heads, head h's scores go to list (layer, h)
};
hipError_t launch_pool_query(const ScoreArgs& a, hipStream_t stream);
hipError_t launch_score(const ScoreArgs& a, hipStream_t stream);

struct SelectArgs {
  const float* scores;  // [n_lists][scores_stride]
  int32_t* keep;        // [n_lists][keep_stride]
  int scores_stride, keep_stride;
  int n_lists;          // layers x index sets per layer
  int P, k, T_first, T_cur;
};
hipError_t launch_select(const SelectArgs& a, hipStream_t stream);
// keep = 0..T-1 (nothing pruned) or first ∪ current (k == 0)
hipError_t launch_fill_keep(int32_t* keep, int keep_stride, int n_lists, int T_first, int P, int T_cur,
                            bool keep_middle, hipStream_t stream);

struct RequantArgs {
  CachePool pool;
  Batch b;
  Workspace ws;
  int Tc, n, Tn;  // old cache length, frame tokens, new cache length (= keep length)
  int frame_id;
  // new positions [0, identity_end) keep their cache row (first frame, or everything cached when nothing is pruned),
  // positions [Tn - n, Tn) are the frame's rows; only the positions in between are looked up in the keep list
  int identity_end;
  // the leading stable_blocks blocks of 64 positions hold the same cached rows as before the step (whole blocks inside
  // [0, identity_end)): such a block is re-quantized from what it already holds, and once that reproduces it bit for
  // bit - flagged per (layer, head, block) by the step that saw it happen - it never changes again and is skipped
  int stable_blocks;
  uint8_t* stable_flag;  // [L][H][Tcap / 64]
  int carry_values;      // xsv_config.value_mode == 1: value rows that come from the cache keep their codes and parameters
};
hipError_t launch_requant(const RequantArgs& a, hipStream_t stream);
hipError_t launch_zero_bytes(uint8_t* p, size_t n, hipStream_t stream);  // a fill kernel (no memset node)

// Canonical (one code per byte, untransposed) copies of one layer buffer → device arrays.
struct UnpackArgs {
  CachePool pool;
  int buf, layer, T;
  uint8_t* k_codes;  // [H][T][64] or null
  float* k_scale;    // [H][ceil(T/G)][64]
  float* k_zero;
  uint8_t* v_codes;
  float* v_scale;  // [H][T][64/G]
  float* v_zero;
  uint16_t* k_bf16;  // [H][T][64] dequantized view / stored rows
  uint16_t* v_bf16;
};
hipError_t launch_unpack(const UnpackArgs& a, hipStream_t stream);

}  // namespace xsv
