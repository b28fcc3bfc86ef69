// Internal declarations shared by the HIP translation units of libgradcomp.
// Not part of the public ABI (that is include/gradcomp.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

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

constexpr int kWaveTile = 1024;   // elements one wave moves per iteration of the streaming pass
constexpr int kSampleGranule = 256;
constexpr int kItemsPerGroup = 4; // one workgroup (4 waves) owns 4 consecutive items of one tensor

enum Mode : int32_t { kDense = 0, kSampled = 1 };

// Immutable per-tensor plan, built on the host, read by every kernel.
struct TensorDesc {
  int64_t off;         // first element in the flat gradient / residual
  int64_t n;           // elements
  int64_t k;           // entries to keep
  int64_t kprefix;     // first output pair of this tensor
  int64_t sprefix;     // first output scale of this tensor
  int64_t item_begin;  // first item (multiple of kItemsPerGroup)
  int64_t item_end;    // one past the last item slot (padded to a multiple of kItemsPerGroup)
  int64_t nitems;      // items that hold elements: ceil(n / item_len)
  int32_t mode;        // Mode
  int32_t sample_len;  // elements sampled from each item (multiple of kSampleGranule)
  uint32_t sample_target;  // sample count that the candidate threshold must cover
  uint32_t pad_;
};

// Per-tensor state of one compress call, zeroed by the first kernel of the call.
struct TensorState {
  unsigned long long cand_total;  // candidates gathered by the streaming pass
  unsigned long long k_rem;       // rank still to resolve inside `prefix`; after the last level: tie quota
  uint32_t t_lo;                  // candidate threshold key (sampled tensors)
  uint32_t overflow;              // some item ran out of candidate slots
  uint32_t prefix;                // resolved high bits of the threshold key; after the last level: T
  uint32_t pad_;
};

struct Workspace {  // device pointers into the context's scratch
  const TensorDesc* td;
  TensorState* ts;
  unsigned long long* shist;  // [T][kSampleBins]
  unsigned long long* hist;   // [T][kSelBins]
  uint32_t* item_cnt;         // candidates per item
  uint32_t* item_gt;          // per item: entries above the threshold
  uint32_t* item_eq;          // per item: entries equal to the threshold
  long long* item_goff;       // exclusive prefix of item_gt within the tensor
  long long* item_eoff;       // exclusive prefix of item_eq within the tensor
  float* cand_val;            // [items][cap]
  uint32_t* cand_rel;         // [items][cap] offset of the candidate inside its item
  float* kept_val;            // [sum k] accumulated values of the kept entries, ascending
  uint32_t* flags;            // [0] non-finite seen
  int32_t T;
  int32_t item_len;
  int32_t cap;
  int32_t pad_;
  int64_t nitem_slots;        // padded item slots over all tensors
};

struct OutBuf {
  void* indices;
  int8_t* q;
  float* scales;
  int32_t index_bits;
  int32_t block;
};

// kernel ids for profiling
enum KernelId : int32_t {
  kKInit = 0, kKSample, kKSampleThresh, kKMain, kKHist, kKSelectScan, kKCount, kKItemScan,
  kKEmit, kKQuant, kKDecBounds, kKDecTiles, kKNum
};

// launchers (defined in the .hip files next to their kernels)
void launch_init(const Workspace& ws, hipStream_t s);
void launch_sample(const Workspace& ws, const void* g, int dtype, const float* e, hipStream_t s);
void launch_sample_thresh(const Workspace& ws, hipStream_t s);
void launch_main(const Workspace& ws, const void* g, int dtype, float* e, hipStream_t s);
void launch_hist(const Workspace& ws, int level, const float* e, hipStream_t s);
void launch_select_scan(const Workspace& ws, int level, hipStream_t s);
void launch_count(const Workspace& ws, const float* e, hipStream_t s);
void launch_item_scan(const Workspace& ws, hipStream_t s);
void launch_emit(const Workspace& ws, const float* e, const OutBuf& out, hipStream_t s);
void launch_quant(const Workspace& ws, float* e, const OutBuf& out, int64_t total_blocks, hipStream_t s);

constexpr int kMaxWorkers = 64;
constexpr int kDecTile = 2048;  // output floats per wave-tile of decompress_sum
struct DecArgs {
  const void* indices[kMaxWorkers];
  const int8_t* q[kMaxWorkers];
  const float* scales[kMaxWorkers];
  uint32_t k[kMaxWorkers];
};
void launch_dec_bounds(const DecArgs& a, int W, int index_bits, int64_t ntiles, uint32_t* bounds,
                       hipStream_t s);
void launch_dec_tiles(const DecArgs& a, int W, int index_bits, int32_t block, int64_t n,
                      int64_t ntiles, const uint32_t* bounds, const long long* kprefix,
                      const long long* sprefix, int T, float* out, hipStream_t s);

}  // namespace gc
