// Internal declarations shared by the HIP translation units of libgradcomp.
// Not part of the public ABI (that is include/gradcomp.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include "gc_fastdiv.h"

namespace gc {

// ---- radix-select geometry ------------------------------------------------
// A key is the 31 magnitude bits of an fp32 pattern. The exact select walks it
// in three digits, most significant first.
constexpr int kSelLevels = 3;
constexpr int kSelBins = 2048;  // histogram bins per tensor (largest digit)
__host__ __device__ constexpr int sel_shift(int level) { return level == 0 ? 20 : (level == 1 ? 9 : 0); }
__host__ __device__ constexpr int sel_bits(int level) { return level == 2 ? 9 : 11; }

// The sampling pre-pass histograms the top 13 key bits (8 exponent + 5 mantissa).
constexpr int kSampleBits = 13;
constexpr int kSampleBins = 1 << kSampleBits;
constexpr int kSampleShift = 31 - kSampleBits;
constexpr int kSampleGranule = 256;  // one wavefront, one 128-bit load per lane and array

// Streaming pass: one workgroup of 4 wavefronts streams one GROUP of consecutive elements once
// (kRows 128-bit loads per lane and array) and exits. With non-temporal loads on both inputs,
// 1024-element groups (one load per lane and array) measured fastest on the 1.3B and 7B
// workloads, 2048- and 4096-element groups 1-3 % slower overall.
#ifndef GC_ROWS
#define GC_ROWS 1
#endif
constexpr int kRows = GC_ROWS;
constexpr int kWaveTile = kRows * 256;
constexpr int kGroup = 4 * kWaveTile;
#ifndef GC_SLOT_LINE
#define GC_SLOT_LINE 16
#endif
// Candidate records leave a workgroup in multiples of 16 (128 bytes, one L2 line), or of 8 when a
// group has at most 8 slots: two neighbouring groups then share a line, and under the die-aware
// order below they run on the same die at about the same time, so their halves meet in L2.
constexpr int kSlotLine = GC_SLOT_LINE;
// Select / compaction passes read their source in CHUNKS: 4096 entries per workgroup, 1024 per
// wavefront.
constexpr int kChunk = 1024;
constexpr int kChunkElems = 4 * kChunk;
// Prefix sums over per-group / per-chunk counts are cut into blocks of 1024 counts.
constexpr int kScanBlock = 1024;

enum Mode : int32_t { kDense = 0, kSampled = 1 };

// Small tensors: one workgroup finishes the tensor after the streaming pass (candidate gather,
// exact select, ordered emit, codes, residual) in ONE launch instead of the chain of a dozen
// grid-wide kernels, whose launch gaps dominate when there is little to do. A sampled tensor
// qualifies with at most kSmallMaxK kept entries and kSmallMaxN elements (the bound on what the one
// workgroup re-reads if the candidates turn out unusable), a tensor selected from its residual
// directly with at most kSmallMaxDenseN elements.
constexpr int64_t kSmallMaxK = 12288;         // candidates (about 1.2 k) then fit the LDS of the one workgroup
constexpr int64_t kSmallMaxN = 4096 * 1024 - 4;   // at most 4096 groups
constexpr int64_t kSmallMaxDenseN = 65536;
#ifndef GC_FINISH_THREADS
#define GC_FINISH_THREADS 1024
#endif
constexpr int kFinishThreads = GC_FINISH_THREADS;

// Immutable per-tensor plan, built on the host, read by every kernel.
struct TensorDesc {
  int64_t off;          // first element in the flat gradient / residual
  int64_t n;            // elements
  int64_t k;            // entries to keep
  int64_t kprefix;      // first output pair of this tensor
  int64_t sprefix;      // first output scale of this tensor
  int64_t qprefix;      // first code byte of this tensor (sign code; equals kprefix for int8)
  int64_t group_begin;  // first group slot of this tensor
  int64_t ngroups;      // ceil(n / kGroup)
  int64_t cand_begin;   // first entry of this tensor's region in the dense candidate arrays
  int64_t cand_cap;     // entries in that region
  int64_t sgran_begin;  // first sampled-granule work item of this tensor
  int64_t nsgran;       // sampled granules
  int32_t mode;         // Mode
  int32_t sample_stride;   // one granule out of this many is sampled
  uint32_t sample_target;  // sample count that the candidate threshold must cover
  int32_t group_shift;     // elements by which the tensor's first group is shortened (0..3)
  int32_t small;           // 1: everything after the streaming pass is done by one workgroup (k_finish)
  int32_t pad_;
};

// Per-tensor state of one compress call, zeroed by the first kernel of the call.
struct TensorState {
  unsigned long long k_rem;  // rank still to resolve inside `prefix`; after the last level: tie quota
  long long vlen;            // entries of the select source: candidates, or n on the dense route
  long long achunk_begin;    // first active chunk of this tensor in the call-wide chunk numbering
  long long cand_total;      // candidates gathered by the streaming pass
  uint32_t t_lo;             // candidate threshold key (sampled tensors)
  uint32_t tie_hint;         // key that may be the threshold with a huge tie (kNoTieHint: none); see tie_spec_count
  uint32_t prefix;           // resolved high bits of the threshold key; after the last level: T
  uint32_t use_cand;         // 1: select from the gathered candidates, 0: from the dense residual
  uint32_t resolved;         // 1: the hinted key was verified as the threshold, the digit passes are skipped
  uint32_t pad_;
};
constexpr uint32_t kNoTieHint = 0xFFFFFFFFu;

// One record per group of the streaming pass (only built when a call has several tensors).
struct GroupRec {
  long long start;   // first element of the group in the flat arrays
  int32_t len;       // elements in the group (1..kGroup)
  uint32_t tensor;   // tensor index; bit 31 set when the tensor is sampled
};

struct Workspace {  // device pointers into the context's scratch
  const TensorDesc* td;             // null for a single-tensor call: its plan travels in td1
  TensorDesc td1;                   // the only tensor's plan, by kernel argument (no upload, no plan cache)
  __host__ __device__ const TensorDesc& desc(int t) const { return td ? td[t] : td1; }
  const GroupRec* recs;       // null when the call has a single tensor
  TensorState* ts;
  unsigned long long* shist;  // [T][kSampleBins]
  unsigned long long* hist;   // [T][kSelBins]
  // streaming pass output
  uint32_t* grp_cnt;                // [groups] candidates of each group (may exceed cap)
  unsigned long long* grp_part;     // [ceil(groups / kScanBlock)] block sums of grp_cnt
  long long* grp_off;               // [groups] exclusive prefix of grp_cnt (call-wide)
  long long* tg_base;               // [T + 1] grp_off at each tensor's first group; [T] = total
  uint2* slots;                     // [groups][slot_stride] records {acc bits, offset inside the group};
                                    // a group writes min(count, cap) of them, none when it has none
  // dense candidate arrays (per-tensor regions)
  float* cand_val;
  long long* cand_idx;              // element index inside the tensor
  // select / compaction over chunks of the source
  uint32_t* ch_gt;                  // [active chunk] entries above the threshold
  uint32_t* ch_eq;                  // [active chunk] entries equal to the threshold
  unsigned long long* ch_part_gt;   // block sums of ch_gt
  unsigned long long* ch_part_eq;
  long long* ch_goff;               // exclusive prefixes (call-wide)
  long long* ch_eoff;
  long long* tb_g;                  // [T] ch_goff at each tensor's first active chunk
  long long* tb_e;
  long long* totals;                // [0] active chunks of the call
  float* kept_val;                  // [sum k] accumulated values of the kept entries, ascending
  uint32_t* flags;                  // [0] non-finite seen
  int32_t T;
  int32_t block;                    // kept entries per quantization block
  int32_t cap;                      // candidate slots per group
  int32_t slot_stride;              // records reserved per group (= cap: 8, or a multiple of 16)
  int32_t gather_team;              // lanes per group in the gather (1 or 16)
  int64_t ngroups;                  // group slots over all tensors
  int64_t nsgran;                   // sampled granules over all tensors
  int64_t max_chunks;               // capacity of the per-chunk arrays
  int64_t n_single;                 // elements of the only tensor (single-tensor calls)
  int64_t nblocks;                  // quantization blocks over all tensors
  int32_t max_chunk_wgs;            // chunks of the call on the dense route: the grid of the chunk kernels is
                                    // sized for it (they grid-stride; workgroups without a chunk leave at once)
  int32_t main_lds_pad;             // dynamic LDS bytes of the streaming pass (occupancy control)
};

struct OutBuf {
  void* indices;
  int8_t* q;
  float* scales;
  int32_t index_bits;
  int32_t block;
  int32_t codec;
};

// kernel ids for profiling
enum KernelId : int32_t {
  kKSample = 0, kKSampleThresh, kKMain, kKGroupSums, kKGroupScan, kKRoute, kKGather, kKHist,
  kKSelectScan, kKCount, kKChunkSums, kKChunkScan, kKEmit, kKQuant, kKFinish, kKDecPack, kKDecTiles, kKDecFused, kKDense, kKDenseSum, kKRowsGather, kKRowsFinish, kKRowsRemap, kKNum
};

// launchers (defined in the .hip files next to their kernels)
void launch_sample(const Workspace& ws, const void* g, int dtype, const float* e, hipStream_t s);
void launch_sample_thresh(const Workspace& ws, hipStream_t s);
void launch_main(const Workspace& ws, const void* g, int dtype, float* e, hipStream_t s);
void launch_group_sums(const Workspace& ws, hipStream_t s);
void launch_chunk_sums(const Workspace& ws, hipStream_t s);
void launch_group_scan(const Workspace& ws, hipStream_t s);
void launch_route(const Workspace& ws, hipStream_t s);
void launch_gather(const Workspace& ws, const float* e, hipStream_t s);
void launch_hist(const Workspace& ws, int level, const float* e, hipStream_t s);
void launch_select_scan(const Workspace& ws, int level, hipStream_t s);
void launch_count(const Workspace& ws, const float* e, hipStream_t s);
void launch_chunk_scan(const Workspace& ws, hipStream_t s);
void launch_emit(const Workspace& ws, const float* e, const OutBuf& out, hipStream_t s);
void launch_quant(const Workspace& ws, float* e, const OutBuf& out, int64_t ktotal, hipStream_t s);
void launch_finish(const Workspace& ws, float* e, const OutBuf& out, hipStream_t s);

// ---- die-aware order of one-shot workgroups ---------------------------------
// Workgroup b runs on compute die b % 8. Work item number xcd_run_index(b) makes every die walk
// runs of kXcdRun consecutive items: 256 items (1 MB per fp32 array for 1024-element items)
// measured best for the streaming pass on the 7B workload (12.71 ms against 12.80 ms for the plain
// order with the operands at the same addresses; runs of 64 items: 12.87, of 16: 14.7 ms). The
// launch grid must be padded with xcd_run_grid().
#ifndef GC_XCD_RUN
#define GC_XCD_RUN 256
#endif
constexpr int kXcds = 8;
constexpr int kXcdRun = GC_XCD_RUN;
__host__ __device__ inline int64_t xcd_run_grid(int64_t items, int64_t run = kXcdRun) {
  const int64_t round = (int64_t)kXcds * run;
  return (items + round - 1) / round * round;
}
__device__ __forceinline__ int64_t xcd_run_index(int64_t b, int64_t run = kXcdRun) {
  const int64_t x = b % kXcds, l = b / kXcds;
  return ((l / run) * kXcds + x) * run + (l % run);
}
// Run length that gives a die about kXcdRun * 1024 consecutive elements at a time.
__host__ __device__ inline int xcd_run_for(int64_t elems_per_item) {
  const int64_t r = (int64_t)kXcdRun * 1024 / (elems_per_item > 0 ? elems_per_item : 1);
  return (int)(r < 1 ? 1 : r);
}

// ---- small device helpers shared by the kernels ----------------------------
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t mbcnt64(uint64_t m) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}
__device__ __forceinline__ uint32_t key_of(float x) { return __float_as_uint(x) & 0x7FFFFFFFu; }

// x / d for the divisor behind f (gc_fastdiv.h): a multiplication and two shifts.
__device__ __forceinline__ uint32_t fast_div(uint32_t x, FastDiv f) {
  const uint32_t t = __umulhi(f.m, x);
  return (t + ((x - t) >> f.s1)) >> f.s2;
}

template <typename G> __device__ __forceinline__ float load_grad(const G* g, int64_t i);
template <> __device__ __forceinline__ float load_grad<float>(const float* g, int64_t i) { return g[i]; }
template <> __device__ __forceinline__ float load_grad<uint16_t>(const uint16_t* g, int64_t i) {
  return __uint_as_float((uint32_t)g[i] << 16);  // bf16 -> fp32 is exact
}

template <typename G> struct GradVec;
template <> struct GradVec<float> {
  static __device__ __forceinline__ f32x4 load(const float* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
  }
  static constexpr uint32_t kAlignMask = 15u;
};
template <> struct GradVec<uint16_t> {
  static __device__ __forceinline__ f32x4 load(const uint16_t* p) {
    const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
    f32x4 r;
    r.x = __uint_as_float(v.x << 16);
    r.y = __uint_as_float(v.x & 0xFFFF0000u);
    r.z = __uint_as_float(v.y << 16);
    r.w = __uint_as_float(v.y & 0xFFFF0000u);
    return r;
  }
  static constexpr uint32_t kAlignMask = 7u;
};

constexpr int kMaxWorkers = 64;
struct DecArgs {
  const void* indices[kMaxWorkers];
  const int8_t* q[kMaxWorkers];
  const float* scales[kMaxWorkers];
  uint32_t k[kMaxWorkers];
  float denom[kMaxWorkers];  // 1 + staleness of the worker (weighted aggregate)
};
constexpr int kDecMinTileShift = 12;  // the smallest output tile of the aggregate: 4096 floats
// log2 of the output tile (floats) for a call, and tiles per range of the packing pass.
int dec_tile_shift(int64_t nrec, int64_t n);
int dec_tile_shift_of(bool large);
int dec_range_tiles(int W, int tshift, int64_t nrec, int64_t n);
// rec: one 8-byte record per pair of all workers; tile_start: ntiles + 1 entries. The packing pass
// takes ranges [r_first, r_first + r_count), the tile pass tiles [t_begin, t_end).
void launch_dec_pack(const DecArgs& a, int W, int index_bits, int tb, int tshift, int32_t block, int64_t ntiles,
                     int64_t r_first, int64_t r_count, const long long* kprefix, const long long* sprefix,
                     const long long* qprefix, int T, int codec, int weighted, void* rec, unsigned long long* tile_start,
                     hipStream_t s);
// The aggregate in one kernel, without the record stream. kprefix / sprefix / qprefix: per-tensor
// prefix tables of multi-tensor buffers (T > 1), else null.
void launch_dec_fused(const DecArgs& a, int W, int index_bits, int32_t block, int codec, int weighted, int64_t n,
                      const long long* kprefix, const long long* sprefix, const long long* qprefix, int T, float* out,
                      int apply, float c_apply, int crowded, hipStream_t s);
void launch_dec_tiles(const void* rec, const unsigned long long* tile_start, uint64_t nrec, int tshift, int64_t n,
                      int64_t t_begin, int64_t t_end, float* out, int apply, float c_apply, unsigned apply_dense_min,
                      hipStream_t s);

// ---- dense codes (every entry kept, no indices) -----------------------------
constexpr int kDenseMaxBlock = 8192;   // larger blocks do not fit one workgroup's registers
struct DenseDecArgs {
  const int8_t* q[kMaxWorkers];
  const float* scales[kMaxWorkers];
  float denom[kMaxWorkers];
};
// idx may be null (no index list); otherwise 0..n-1 is written with `index_bits` wide entries.
// Blocks of up to wave_block (<= 2048) elements are owned by one wavefront, larger ones by the workgroup;
// lds_pad bytes of dynamic LDS only bound how many workgroups share a compute unit.
void launch_dense(const void* g, int dtype, float* e, int64_t n, int32_t block, int codec, void* q,
                  float* scales, void* idx, int index_bits, uint32_t* flags, int wave_block, int lds_pad,
                  hipStream_t s);
void launch_dense_sum(const DenseDecArgs& a, int W, int32_t block, int64_t n, int codec, float* out,
                      int weighted, int apply, float c_apply, hipStream_t s);

// ---- row-sparse gradients (touched rows of a table-shaped residual) ----------
void launch_rows_gather(const float* table, const long long* rows, int64_t U, int64_t D, int64_t R, float* ec,
                        uint32_t* flags, hipStream_t s);
struct RowsRemapArgs {  // every worker's index list for the one launch that rewrites them all
  const void* idx[kMaxWorkers];
  uint32_t k[kMaxWorkers];
  uint32_t at[kMaxWorkers];   // first compact position of the worker in the output
  uint8_t bits[kMaxWorkers];  // 32 or 64
};
void launch_rows_remap(const RowsRemapArgs& a, int W, const long long* urows, int64_t Ru, int64_t D, uint32_t* out,
                       uint32_t* flags, hipStream_t s);
void launch_rows_finish(float* table, const long long* rows, int64_t U, int64_t D, int64_t R, const float* ec,
                        const uint32_t* compact_idx, int64_t k, void* out_idx, int index_bits, hipStream_t s);

}  // namespace gc
