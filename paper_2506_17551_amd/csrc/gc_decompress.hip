// Decompress-and-sum: the aggregate of W workers' compressed gradients as a dense
// fp32 vector (paper Sec. III.B, Eq. 8 without the 1/P), for gfx950.
//
// The workers' pairs arrive as W separate sorted lists (3 arrays each). Reading them tile by tile
// means dozens of short reads from as many arrays per tile, which bounds the kernel by memory
// latency, not by the 4 bytes per element it has to write. So the pairs are first merged into ONE
// stream that is already in the order the tiles consume it:
//
//   k_dec_pack      one workgroup per range of `tb` output tiles: finds every worker's first pair
//                   in the range and after it (binary search in the worker's ascending index list),
//                   then, in LDS, where every (tile, worker) segment starts, decodes the range's
//                   pairs (coalesced reads along each worker's list) and writes them as 8-byte
//                   records {position in tile | worker << 16, value}, ordered by tile, then worker,
//                   then index. tile_start[t] is the first record of tile t. All of a range's
//                   records lie in one window of the stream.
//   k_dec_tiles     one wavefront per tile of output floats held in LDS (4096 floats; 16384 where
//                   tiles are thinly filled, see dec_tile_shift): reads the
//                   tile's run of records with coalesced loads, adds them into the LDS tile worker
//                   by worker (ascending), then writes the tile once with 128-bit stores. Every
//                   output byte is written exactly once; there is no separate memset and no global
//                   atomic. Indices are unique inside one worker's buffer, so the adds of one
//                   worker never collide, and the fixed worker order makes the fp32 sum
//                   reproducible bit for bit.
//
// Up to 32 workers the call takes k_dec_fused (further down) instead: one kernel that reads a
// tile's pairs straight from the workers' lists and never writes the merged stream.
//
// Index lists that break the contract (not ascending, duplicates, out of range) give an unspecified
// sum, but every access stays inside the caller's and the library's arrays: records are only
// written inside their segment, and positions and workers read back from records are range-checked.
#include "gc_internal.h"

namespace gc {
namespace {


template <typename I>
__device__ __forceinline__ uint32_t lower_bound_idx(const I* __restrict__ idx, uint32_t lo, uint32_t hi,
                                                    unsigned long long target) {
  while (lo < hi) {  // first j in [lo, hi] with idx[j] >= target
    const uint32_t mid = lo + ((hi - lo) >> 1);
    if ((unsigned long long)idx[mid] < target) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// lower_bound by eight lanes at a time: every step probes eight positions that cut [lo, hi) into
// nine pieces, so the chain of dependent loads is 8 deep instead of 23 for a list of 7 M indices.
// All eight lanes of a group (consecutive lanes, group g = lane / 8) call it with the same arguments
// and get the same result; lanes of a group with nothing to search pass hi = 0.
template <typename I>
__device__ __forceinline__ uint32_t lower_bound_idx8(const I* __restrict__ idx, uint32_t hi, unsigned long long target,
                                                     int lane) {
  const int sub = lane & 7, gsh = lane & ~7;
  uint32_t lo = 0u;
  while (__ballot(lo < hi) != 0ull) {  // the wavefront leaves together: the ballots below need every lane
    const uint32_t width = hi > lo ? hi - lo : 0u;
    const uint32_t stepw = width / 9u + 1u;
    const uint32_t p = lo + (uint32_t)(sub + 1) * stepw - 1u;  // probe position of this lane
    bool less = false;
    if (lo < hi && p < hi) less = (unsigned long long)idx[p] < target;
    const uint32_t field = (uint32_t)((__ballot(less) >> gsh) & 0xFFull);  // sorted list: the true lanes are a prefix
    const uint32_t c = (uint32_t)__popc(field);
    if (lo < hi) {
      const uint32_t nlo = lo + c * stepw;                 // one past the last probe that was below the target
      const uint32_t nhi_p = lo + (c + 1u) * stepw - 1u;   // the first probe at or above it
      if (c < 8u && nhi_p < hi) hi = nhi_p;
      lo = nlo < hi ? nlo : hi;
    }
  }
  return lo;
}

// The wavefronts of a workgroup share out the workers (several wavefronts per worker when there are
// few workers); every lane issues the loads of a batch of pairs before it uses any of them.
#ifndef GC_PACK_THREADS
#define GC_PACK_THREADS 256
#endif
#ifndef GC_PACK_BATCH
#define GC_PACK_BATCH 4
#endif
constexpr int kPackThreads = GC_PACK_THREADS, kPackWaves = kPackThreads / 64;
constexpr int kPackBatch = GC_PACK_BATCH;  // pairs per lane whose loads are issued before any is used

template <typename I>
__global__ __launch_bounds__(kPackThreads) void k_dec_pack(DecArgs a, int W, int tb, int tshift, int32_t block, FastDiv bdiv,
                                                           int64_t ntiles,
                                                           int64_t r_first,
                                                           const long long* __restrict__ kprefix,
                                                           const long long* __restrict__ sprefix,
                                                           const long long* __restrict__ qprefix, int T, int codec,
                                                           int weighted, uint2* __restrict__ rec,
                                                           unsigned long long* __restrict__ tile_start) {
  extern __shared__ uint32_t s_dyn[];
  uint32_t* s_lo = s_dyn;                  // [tb + 1][W]: first pair of worker w at or after local tile t
  uint32_t* s_off = s_dyn + (tb + 1) * W;  // [tb][W]: first record of segment (t, w) inside the range
  __shared__ uint32_t s_br0[kMaxWorkers], s_excl[kMaxWorkers + 1], s_wave[kPackThreads / 64];
  __shared__ unsigned long long s_base;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int team = W >= kPackWaves ? 1 : kPackWaves / W;  // wavefronts that share one worker's pairs
  const unsigned long long step = 64ull * team;
  const int64_t r = r_first + blockIdx.x, t0 = r * tb;

  // every worker's first pair at or after the start of this range and of the next one: 2 W lower
  // bounds, eight lanes each (8 dependent loads instead of 23 for a list of 7 M indices)
  __shared__ uint32_t s_br1[kMaxWorkers];
  for (int s0 = 0; s0 < 2 * W; s0 += kPackThreads / 8) {
    const int sidx = s0 + tid / 8;
    const bool on = sidx < 2 * W;
    const int w = on ? (sidx < W ? sidx : sidx - W) : 0;
    const unsigned long long target = ((unsigned long long)(r + (sidx < W ? 0 : 1)) * (unsigned long long)tb) << tshift;
    const uint32_t b = lower_bound_idx8<I>(static_cast<const I*>(a.indices[w]), on ? a.k[w] : 0u, target, lane);
    if (on && (tid & 7) == 0) {
      if (sidx < W) s_br0[w] = b; else s_br1[w] = b;
    }
  }
  __syncthreads();
  if (tid < W) {
    const uint32_t b0 = s_br0[tid], b1 = s_br1[tid];
    s_excl[tid + 1] = b1 > b0 ? b1 - b0 : 0u;  // count, turned into a prefix below
  }
  __syncthreads();
  if (tid == 0) {
    unsigned long long base = 0ull;  // records before this range: every worker's pairs before it
    uint32_t run = 0u;
    for (int w = 0; w < W; ++w) {
      const uint32_t c = s_excl[w + 1];
      base += s_br0[w];
      s_excl[w] = run;
      run += c;
    }
    s_excl[W] = run;
    s_base = base;
  }
  __syncthreads();
  const uint32_t total = s_excl[W];
  for (int i = tid; i < (tb + 1) * W; i += kPackThreads) {  // a tile after a worker's last pair starts at its end
    const int w = i % W;
    s_lo[i] = s_br0[w] + (s_excl[w + 1] - s_excl[w]);
  }
  __syncthreads();

  // the first pair at or after the start of every tile: pair j opens all tiles after its predecessor's, up to its own
  for (int w = wave / team; w < W; w += kPackWaves / team) {
    const I* idx = static_cast<const I*>(a.indices[w]);
    const unsigned long long j0 = s_br0[w], j1 = j0 + (s_excl[w + 1] - s_excl[w]);  // 64 bits: j1 may sit just below 2^32
    for (unsigned long long jb = j0 + (unsigned)((wave % team) * 64 + lane); jb < j1; jb += step * kPackBatch) {
      unsigned long long cur[kPackBatch], prev[kPackBatch];
#pragma unroll
      for (int u = 0; u < kPackBatch; ++u) {  // the batch's loads are in flight together
        const unsigned long long j = jb + u * step;
        cur[u] = 0ull;
        prev[u] = 0ull;
        if (j < j1) {
          cur[u] = (unsigned long long)idx[j];
          if (j > j0) prev[u] = (unsigned long long)idx[j - 1];
        }
      }
#pragma unroll
      for (int u = 0; u < kPackBatch; ++u) {
        const unsigned long long j = jb + u * step;
        const int64_t tc = (int64_t)(cur[u] >> tshift) - t0;
        if (j < j1 && tc >= 0 && tc < tb) {  // outside only with indices out of order
          int64_t tp = -1;
          if (j > j0) {
            tp = (int64_t)(prev[u] >> tshift) - t0;
            if (tp < -1) tp = -1;
          }
          for (int64_t t = tp + 1; t <= tc; ++t) s_lo[t * W + w] = (uint32_t)j;
        }
      }
    }
  }
  __syncthreads();

  // exclusive scan of the segment lengths in (tile, worker) order
  const int nent = tb * W, per = (nent + kPackThreads - 1) / kPackThreads;
  const int beg = tid * per, end = beg + per < nent ? beg + per : nent;
  uint32_t sum = 0u;
  for (int i = beg; i < end; ++i) {
    const uint32_t l0 = s_lo[i], l1 = s_lo[i + W];
    sum += l1 > l0 ? l1 - l0 : 0u;
  }
  uint32_t incl = sum;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t u = __shfl_up(incl, off);
    if (lane >= off) incl += u;
  }
  if (lane == 63) s_wave[wave] = incl;
  __syncthreads();
  uint32_t run = incl - sum;
  for (int x = 0; x < wave; ++x) run += s_wave[x];
  for (int i = beg; i < end; ++i) {
    const uint32_t l0 = s_lo[i], l1 = s_lo[i + W];
    s_off[i] = run;
    run += l1 > l0 ? l1 - l0 : 0u;
  }
  __syncthreads();

  // the range also writes where it ends (the next range writes the same number there as its own
  // start): the tiles of this range can then be consumed before the next range has been packed
  for (int t = tid; t <= tb; t += kPackThreads)
    if (t0 + t <= ntiles) tile_start[t0 + t] = s_base + (t < tb ? s_off[t * W] : total);

  for (int w = wave / team; w < W; w += kPackWaves / team) {
    const I* idx = static_cast<const I*>(a.indices[w]);
    const int8_t* qw = a.q[w];
    const float* scw = a.scales[w];
    const float denom = a.denom[w];
    const unsigned long long j0 = s_br0[w], j1 = j0 + (s_excl[w + 1] - s_excl[w]);
    for (unsigned long long jb = j0 + (unsigned)((wave % team) * 64 + lane); jb < j1; jb += step * kPackBatch) {
      unsigned long long gi[kPackBatch];
      float val[kPackBatch];
#pragma unroll
      for (int u = 0; u < kPackBatch; ++u) {  // index, scale and code of the whole batch are in flight together
        const unsigned long long j = jb + u * step;
        gi[u] = 0ull;
        val[u] = 0.0f;
        if (j < j1) {
          gi[u] = (unsigned long long)idx[j];
          uint32_t rel = (uint32_t)j;  // pair inside its tensor; sbase, qbase: the tensor's first scale and code byte
          long long sbase = 0, qbase = 0;
          if (T > 1) {  // blocks restart at every tensor: find the tensor that owns pair j
            int tl = 0, th = T - 1;
            while (tl < th) {
              const int mid = (tl + th + 1) >> 1;
              if (kprefix[mid] <= (long long)j) tl = mid; else th = mid - 1;
            }
            rel = (uint32_t)((long long)j - kprefix[tl]);
            sbase = sprefix[tl];
            qbase = qprefix[tl];
          }
          const uint32_t blk = fast_div(rel, bdiv);
          const float sc = scw[sbase + blk];
          if (codec == 0) {
            val[u] = __fmul_rn((float)qw[qbase + rel], sc);
          } else {  // sign code (Eq. 10): bit number rel - blk * block of the block's bytes
            const uint32_t bit = rel - blk * (uint32_t)block;
            const uint32_t byte = (uint8_t)qw[qbase + (long long)blk * ((block + 7) / 8) + (bit >> 3)];
            val[u] = ((byte >> (bit & 7u)) & 1u) ? sc : -sc;
          }
          if (weighted) val[u] = __fdiv_rn(val[u], denom);  // Eq. 12: a stale worker counts for less
        }
      }
#pragma unroll
      for (int u = 0; u < kPackBatch; ++u) {
        const unsigned long long j = jb + u * step;
        const int64_t tc = (int64_t)(gi[u] >> tshift) - t0;
        if (j < j1 && tc >= 0 && tc < tb) {
          const uint32_t lo = s_lo[tc * W + w], hi = s_lo[(tc + 1) * W + w];
          const uint32_t dest = s_off[tc * W + w] + ((uint32_t)j - lo);
          // a record is only written inside its own segment (it always is when the indices ascend)
          if ((uint32_t)j >= lo && (uint32_t)j < hi && dest < total) {
            const uint32_t pos = (uint32_t)(gi[u] - ((unsigned long long)(t0 + tc) << tshift));
            rec[s_base + dest] = make_uint2(pos | ((uint32_t)w << 16), __float_as_uint(val[u]));
          }
        }
      }
    }
  }
}

// Tiles of 4096 floats (16 KB of LDS per wavefront, 8 wavefronts per workgroup), or of 16384 floats
// (64 KB, 2 wavefronts) where a tile of 4096 would hold few records: with large tiles the long
// vectors at low density (7B at 0.1 %, 16 workers: 66 records per 4096 floats) spend less per tile
// on everything but the write (5.35 against 5.8 ms), while crowded tiles (1.3B at 0.5 %: 330
// records) do better small (1.2 against 2.0 ms). One persistent workgroup per compute unit.
constexpr int kDecTileShiftSmall = kDecMinTileShift, kDecWavesSmall = 8;
constexpr int kDecTileShiftLarge = 14, kDecWavesLarge = 2;
constexpr int kDecGrid = 256;
static_assert(kDecTileShiftLarge <= 16, "a record keeps the position in 16 bits");
static_assert(kMaxWorkers <= 65536, "a record keeps the worker in 16 bits");
constexpr int kDecRounds = 4;            // rounds of 64 records whose loads are in flight together

constexpr uint32_t kClaimed = 0x7FC0DEADu;   // a NaN pattern no finite sum can produce
constexpr uint32_t kNoRecord = 0xFFFFFFFFu;  // position 0xFFFF: outside every tile

__device__ __forceinline__ void wave_sync() {  // orders the wavefront's own LDS accesses
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// Adds one round of records into the wavefront's LDS tile so that equal positions of different
// workers are added in ascending worker order (the records of a tile are in worker order): one LDS
// float add (round to nearest even, denormals kept, like the plain fp32 add) per worker present in
// the round, issued back to back. The LDS executes a wavefront's instructions in the order they
// were issued, so nothing has to wait in between, and within one worker the positions are unique,
// so the lanes of one instruction never collide.
template <int TILE>
__device__ __forceinline__ void add_round(uint2 r, float* lt) {
  const uint32_t pos = r.x & 0xFFFFu;
  const int w = (int)((r.x >> 16) < (uint32_t)(kMaxWorkers - 1) ? (r.x >> 16) : (uint32_t)(kMaxWorkers - 1));
  const bool act = pos < (uint32_t)TILE;
  const uint64_t am = __ballot(act);
  if (am == 0ull) return;
  const int w_first = __builtin_amdgcn_readlane(w, __ffsll((unsigned long long)am) - 1);
  const int w_last = __builtin_amdgcn_readlane(w, 63 - __clzll((unsigned long long)am));
  const float val = __uint_as_float(r.y);
  for (int x = w_first; x <= w_last; ++x) {
    if (act && w == x) (void)__hip_atomic_fetch_add(lt + pos, val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
    __builtin_amdgcn_wave_barrier();  // keeps the instructions in this order
  }
}

// MODE 0: out[tile] = sum (dense write).  MODE 1: theta[i] -= c * sum[i] at the touched i only.
// Wavefronts walk the tiles with a grid stride, without workgroup barriers.
template <int MODE, int TILE, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void k_dec_tiles(const uint2* __restrict__ rec,
                                                   const unsigned long long* __restrict__ tile_start,
                                                   unsigned long long nrec, int64_t n, int64_t t_begin,
                                                   int64_t t_end, float* __restrict__ out, float c_apply,
                                                   unsigned apply_dense_min) {
  __shared__ float tile_mem[WAVES][TILE];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  float* lt = tile_mem[wave];
  const int64_t stride = (int64_t)gridDim.x * WAVES;

  for (int64_t tile = t_begin + (int64_t)blockIdx.x * WAVES + wave; tile < t_end; tile += stride) {
    const int64_t base = tile * TILE;
    unsigned long long first = tile_start[tile], last = tile_start[tile + 1];
    if (last > nrec) last = nrec;
    const unsigned long long total = last > first ? last - first : 0ull;
    if (MODE == 1 && total == 0ull) continue;  // nothing to apply in an empty tile

    const f32x4 z = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int i = 0; i < TILE / 256; ++i) *reinterpret_cast<f32x4*>(lt + (i * 64 + lane) * 4) = z;
    wave_sync();

    for (unsigned long long s0 = 0; s0 < total; s0 += 64 * kDecRounds) {
      uint2 r[kDecRounds];
#pragma unroll
      for (int i = 0; i < kDecRounds; ++i) {
        const unsigned long long p = s0 + (unsigned long long)(i * 64 + lane);
        r[i] = make_uint2(kNoRecord, 0u);
        if (p < total) r[i] = rec[first + p];
      }
#pragma unroll
      for (int i = 0; i < kDecRounds; ++i) add_round<TILE>(r[i], lt);
    }
    wave_sync();

    if (MODE == 0) {
      const int64_t remain = n - base;
      if (remain >= TILE && ((reinterpret_cast<uintptr_t>(out) & 15u) == 0)) {
#pragma unroll
        for (int i = 0; i < TILE / 256; ++i) {
          const f32x4 v = *reinterpret_cast<const f32x4*>(lt + (i * 64 + lane) * 4);
          __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(out + base + (i * 64 + lane) * 4));
        }
      } else {
        const int lim = (int)(remain < TILE ? remain : TILE);
        for (int i = lane; i < lim; i += 64) out[base + i] = lt[i];
      }
    } else if (total >= (unsigned long long)apply_dense_min && n - base >= TILE &&
               ((reinterpret_cast<uintptr_t>(out) & 15u) == 0)) {
      // A crowded tile (about one touched position per 128-byte line of theta, or more) is read and
      // rewritten whole with full-width accesses: scattered 4-byte read-modify-writes move a 32-byte
      // piece each way per position and run at a fraction of the streaming rate. Where nothing was
      // named the sum is +0 and theta - fl32(c * +0) is theta itself, bit for bit.
#pragma unroll 4
      for (int i = 0; i < TILE / 256; ++i) {
        const f32x4 sm = *reinterpret_cast<const f32x4*>(lt + (i * 64 + lane) * 4);
        f32x4* p = reinterpret_cast<f32x4*>(out + base + (i * 64 + lane) * 4);
        f32x4 th = *p;
        th.x = __fsub_rn(th.x, __fmul_rn(c_apply, sm.x));
        th.y = __fsub_rn(th.y, __fmul_rn(c_apply, sm.y));
        th.z = __fsub_rn(th.z, __fmul_rn(c_apply, sm.z));
        th.w = __fsub_rn(th.w, __fmul_rn(c_apply, sm.w));
        *p = th;
      }
    } else {
      // every touched position is claimed once (LDS exchange with a marker) and updated in place:
      // theta - fl32(c * sum). Untouched positions have sum +0 and would not change anyway. The
      // loads of a batch of rounds are all issued before the first store.
      for (unsigned long long s0 = 0; s0 < total; s0 += 64 * kDecRounds) {
        int64_t gi[kDecRounds];
        float sum[kDecRounds], th[kDecRounds];
        bool mine[kDecRounds];
#pragma unroll
        for (int i = 0; i < kDecRounds; ++i) {
          const unsigned long long p = s0 + (unsigned long long)(i * 64 + lane);
          mine[i] = false;
          gi[i] = 0;
          sum[i] = 0.0f;
          if (p < total) {
            const uint32_t pos = rec[first + p].x & 0xFFFFu;
            gi[i] = base + (int64_t)pos;
            if (pos < (uint32_t)TILE && gi[i] < n) {
              const uint32_t old = atomicExch(reinterpret_cast<uint32_t*>(lt) + pos, kClaimed);
              mine[i] = old != kClaimed;
              sum[i] = __uint_as_float(old);
            }
          }
        }
#pragma unroll
        for (int i = 0; i < kDecRounds; ++i) th[i] = mine[i] ? out[gi[i]] : 0.0f;
#pragma unroll
        for (int i = 0; i < kDecRounds; ++i)
          if (mine[i]) out[gi[i]] = __fsub_rn(th[i], __fmul_rn(c_apply, sum[i]));
      }
    }
    wave_sync();
  }
}

// ---------------------------------------------------------------- fused aggregate
// One kernel, no record stream: a workgroup (4 wavefronts) takes a range of `tb` tiles, finds every
// worker's pairs in it (binary searches, then the "pair j opens the tiles up to its own" pass over
// the range's indices, as k_dec_pack does) and keeps the table of (tile, worker) segment starts in
// LDS. Its wavefronts then take the range's tiles one by one: a tile's pairs are read straight from
// the workers' lists, the lanes dealt out over the tile's pairs in (worker, index) order, decoded in
// registers and added into the LDS tile worker by worker, as k_dec_tiles adds records. The merged
// stream of 8-byte records is never written or read back: that stream is 1.8 GB of the 31.9 GB the
// two-kernel call moves at 7B, and a third of what it moves at 1.3B.
//
// A tile is a chain of memory round trips (table, pairs, adds, store), and a compute unit holds only
// 14 or 16 tiles at a time, so the chain is kept short: a lane finds the worker of its pair by
// comparing its flat position with the W segment starts broadcast from registers (no search through
// LDS), the pairs of the wavefront's NEXT tile are requested before the current tile is summed (what
// arrives is kept raw - index, code byte, scale - and decoded when it is used), and the first pass
// over a range's indices keeps 8 or 16 loads per lane in flight.
struct FusedWorker {  // one worker's arrays, copied to LDS so that a lane can index them by its worker
  const void* idx;
  const int8_t* q;
  const float* sc;
  float denom;
  uint32_t k;
};

// Tiles of 2048 floats, one per wavefront, in two shapes. Crowded tiles: two workgroups of 8
// wavefronts per compute unit, all of which prepare a range together and then take its tiles (the
// first pass over a crowded range's indices needs every lane). Thinly filled tiles: one workgroup of
// 14 tile wavefronts and 2 that only prepare the next range, so the 14 never stop writing.
constexpr int kFusedTileShift = 11;
constexpr int kFusedWavesCrowded = 8;
constexpr int kFusedWavesThin = 14, kFusedPrepThin = 2;
constexpr uint32_t kNoPair = 0xFFFFFFFFu;
constexpr int kFusedLdsTensors = 256;  // prefix tables of up to this many tensors are staged in LDS (3 KB)

template <typename I>
struct FusedRaw {  // one pair as it comes out of memory
  I gi;           // global index
  float sc;       // scale of its block
  uint32_t qb;    // its code byte (int8 code, or the byte that holds its sign bit)
  uint32_t aux;   // worker << 16 | bit inside the byte (sign code); kNoPair: no pair in this lane
};

struct FusedTile {  // a tile's segments, one worker per lane
  uint32_t lo;    // first pair of this lane's worker in the tile
  uint32_t cnt;   // and how many
  uint32_t total;
};

// The value held by the lane to the left inside a row of 16 lanes (the first lane of a row keeps its
// own): a shift in the vector unit, without the trip through LDS that a general shuffle takes.
__device__ __forceinline__ uint32_t lane_left(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x111 /* row_shr:1 */, 0xF, 0xF, false);
}
__device__ __forceinline__ unsigned long long lane_left(unsigned long long v) {
  return ((unsigned long long)lane_left((uint32_t)(v >> 32)) << 32) | lane_left((uint32_t)v);
}

// The pairs at flat positions f0 + i * 64 + lane, i < NR, of a tile: worker and pair number. The
// worker of position f is the last one whose segment starts at or before f (an empty segment
// starts where the next one does, and is overruled by it). The segment starts are a running sum of
// the counts, broadcast from the lanes that hold them: scalar work beside NR compares per worker.
template <int NR, int R>
__device__ __forceinline__ void fused_select(const FusedTile& h, int W, uint32_t f0, int lane, int (&ws)[R],
                                             uint32_t (&js)[R]) {
  uint32_t run = 0u;
  for (int w = 0; w < W; ++w) {
    const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)h.cnt, w);
    const uint32_t ad = (uint32_t)__builtin_amdgcn_readlane((int)h.lo, w) - run;
#pragma unroll
    for (int i = 0; i < NR; ++i) {
      const uint32_t f = f0 + (uint32_t)(i * 64 + lane);
      if (f >= run) {
        ws[i] = w;
        js[i] = f + ad;
      }
    }
    run += c;
  }
}

// MODE 0: out[tile] = sum (dense write).  MODE 1: theta[i] -= c * sum[i] at the touched i only.
// PROD > 0 adds that many wavefronts that do nothing but prepare: while the WAVES others sum and
// write the tiles of one range out of one table, they search the brackets of the workgroup's next
// range and fill the other table, each for its own share of the workers and without a word to the
// others, so that the tile wavefronts never stop writing (two tables, one barrier per range). With
// PROD = 0 all wavefronts prepare a range together, then take its tiles.
template <typename I, int MODE, int TSHIFT, int WAVES, int PROD>
__device__ __forceinline__ void dec_fused_body(const DecArgs& a, int W, int tb, int32_t block, FastDiv bdiv, int64_t ntiles,
                                               int64_t nranges, int codec, int weighted, int64_t n,
                                               const long long* __restrict__ kprefix,
                                               const long long* __restrict__ sprefix,
                                               const long long* __restrict__ qprefix, int T,
                                               float* __restrict__ out, float c_apply) {
  // one table, or two with preparing wavefronts, of [tb + 1][W]: first pair of worker w at or after local tile t
  extern __shared__ uint32_t s_dyn[];
  constexpr int kFusedTile = 1 << TSHIFT, kFusedWaves = WAVES, kFusedThreads = (WAVES + PROD) * 64;
  constexpr int kBuild = PROD ? 64 : kFusedThreads;  // threads that prepare a range together
  __shared__ float tile_mem[kFusedWaves][kFusedTile];
  __shared__ FusedWorker s_wk[kMaxWorkers];
  __shared__ uint32_t s_br0[kMaxWorkers], s_br1[kMaxWorkers];
  __shared__ int s_next_tile[2];  // per table: next tile of the range that no wavefront has taken yet
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int btid = PROD ? lane : tid;  // number of this thread among those that prepare together
  const int tab_len = (tb + 1) * W;
  // the workers this thread's group prepares: all of them, or the share of its preparing wavefront
  const int w_per = PROD ? (W + PROD - 1) / PROD : W;
  const int w_begin = PROD ? min(W, max(0, wave - WAVES) * w_per) : 0;
  const int w_end = PROD ? min(W, w_begin + w_per) : W;
  const int Wl = w_end - w_begin;
  constexpr int tshift = TSHIFT;
  constexpr int R = kDecRounds;
  static_assert(R == 4, "fused_select is dispatched for up to four rounds");
  // indices per lane in flight in the first pass: what the register budget of the shape allows
  constexpr int kScan = (WAVES > 4 || PROD) ? 8 : (sizeof(I) == 4 ? 32 : 16);
  // per-tensor prefix tables of a multi-tensor buffer: a pair's tensor is found by a binary search,
  // a chain of dependent reads that is ten times shorter out of LDS than out of memory
  __shared__ uint32_t s_tp[3][kFusedLdsTensors];
  if (T > 1 && T <= kFusedLdsTensors) {
    for (int t = tid; t < T; t += kFusedThreads) {
      s_tp[0][t] = (uint32_t)kprefix[t];
      s_tp[1][t] = (uint32_t)sprefix[t];
      s_tp[2][t] = (uint32_t)qprefix[t];
    }
  }
  if (tid < W) {
    FusedWorker f;
    f.idx = a.indices[tid];
    f.q = a.q[tid];
    f.sc = a.scales[tid];
    f.denom = a.denom[tid];
    f.k = a.k[tid];
    s_wk[tid] = f;
  }
  __syncthreads();
  float* lt = tile_mem[wave < kFusedWaves ? wave : 0];  // the preparing wavefront has no tile
  int G = 64;  // lanes per worker in the first pass over a range's indices
  while (G > 1 && G * Wl > kBuild) G >>= 1;
  const int gl = btid & (G - 1);
  // lanes whose left neighbour is not their predecessor in the worker's list (first of a group), or is
  // out of reach of the row shift (first of a row of 16): they load the predecessor's index themselves
  const bool edge = gl == 0 || (lane & 15) == 0;
  const uint32_t sign_bytes = (uint32_t)((block + 7) / 8);

  // the threads that prepare wait for each other: one wavefront for itself, else the workgroup
  auto build_sync = [&]() {
    if (PROD) wave_sync(); else __syncthreads();
  };
  // ---- prepares range r: its table of segment starts and its tile counter
  auto build = [&](int64_t r, uint32_t* s_lo, int* s_next) {
    const int64_t t0 = r * tb;
    // every worker's first pair at or after the start of this range and of the next one
    for (int s0 = 0; s0 < 2 * Wl; s0 += kBuild / 8) {  // eight lanes per search
      const int s = s0 + btid / 8;
      const bool on = s < 2 * Wl;
      const int w = on ? w_begin + (s < Wl ? s : s - Wl) : 0;
      const unsigned long long target = ((unsigned long long)(r + (s < Wl ? 0 : 1)) * (unsigned long long)tb) << tshift;
      const uint32_t b = lower_bound_idx8<I>(static_cast<const I*>(s_wk[w].idx), on ? s_wk[w].k : 0u, target, lane);
      if (on && (btid & 7) == 0) {
        if (s < Wl) s_br0[w] = b; else s_br1[w] = b;
      }
    }
    build_sync();
    if (btid == 0 && w_begin == 0) *s_next = kFusedWaves;  // tiles 0 .. waves-1 are taken without the counter
    for (int i = btid; i < (tb + 1) * Wl; i += kBuild) {  // a tile after a worker's last pair starts at its end
      const int w = w_begin + i % Wl;
      const uint32_t b0 = s_br0[w], b1 = s_br1[w];
      s_lo[(i / Wl) * W + w] = b1 > b0 ? b1 : b0;
    }
    build_sync();
    // the first pair at or after the start of every tile: pair j opens all tiles after its
    // predecessor's, up to its own. The predecessor's index comes from the lane to the left.
    // Every worker has a group of G consecutive lanes, all workers at once (as many as fit): the
    // whole pass is a few rounds of loads, however many workers there are.
    for (int w0 = w_begin; w0 < w_end; w0 += kBuild / G) {
      const int w = w0 + btid / G;
      const bool wn = w < w_end;
      const I* idx = static_cast<const I*>(s_wk[wn ? w : 0].idx);
      const unsigned long long j0 = wn ? s_br0[w] : 0ull;
      const unsigned long long j1 = wn ? (s_br1[w] > s_br0[w] ? s_br1[w] : s_br0[w]) : 0ull;
      for (unsigned long long jg = j0; __ballot(jg < j1) != 0ull; jg += (unsigned long long)(G * kScan)) {
        I cur[kScan], left[kScan];
        int nu = kScan;  // a short range ends the batch early (uniform over the wavefront)
#pragma unroll
        for (int u = 0; u < kScan; ++u) {  // the batch's loads are in flight together
          const unsigned long long j = jg + (unsigned)(u * G + gl);
          if (u < nu && __ballot(j < j1) == 0ull) nu = u;
          cur[u] = (I)0;
          left[u] = (I)0;
          if (u < nu) {
            cur[u] = j < j1 ? idx[j] : (I)0;
            left[u] = (edge && j < j1 && j > j0) ? idx[j - 1] : (I)0;
          }
        }
#pragma unroll
        for (int u = 0; u < kScan; ++u) {
          if (u >= nu) break;
          const unsigned long long j = jg + (unsigned)(u * G + gl);
          const I from_left = lane_left(cur[u]);  // every lane takes part, also those that will not use it
          const unsigned long long prev = edge ? (unsigned long long)left[u] : (unsigned long long)from_left;
          const int64_t tc = (int64_t)((unsigned long long)cur[u] >> tshift) - t0;
          if (j < j1 && tc >= 0 && tc < tb) {  // outside only with indices out of order
            int64_t tp = -1;
            if (j > j0) {
              tp = (int64_t)(prev >> tshift) - t0;
              if (tp < -1) tp = -1;
            }
            for (int64_t t = tp + 1; t <= tc; ++t) s_lo[t * W + w] = (uint32_t)j;
          }
        }
      }
    }
    build_sync();  // the next search rewrites the brackets
  };

  // ---- the tiles of range r, one wavefront each
  auto consume = [&](int64_t r, const uint32_t* s_lo, int* s_next) {
    const int64_t t0 = r * tb;
    // segments of local tile `ltile`: worker `lane`'s first pair and count
    auto open_tile = [&](int ltile, FusedTile& h) {
      h.lo = 0u;
      h.cnt = 0u;
      if (lane < W) {
        h.lo = s_lo[ltile * W + lane];
        const uint32_t hi = s_lo[(ltile + 1) * W + lane];
        h.cnt = hi > h.lo ? hi - h.lo : 0u;
      }
      uint32_t total = 0u;
      for (int w = 0; w < W; ++w) total += (uint32_t)__builtin_amdgcn_readlane((int)h.cnt, w);
      h.total = total;
    };
    auto select = [&](const FusedTile& h, uint32_t f0, int (&ws)[R], uint32_t (&js)[R]) {
#pragma unroll
      for (int i = 0; i < R; ++i) {
        ws[i] = 0;
        js[i] = 0u;
      }
      const uint32_t left = h.total > f0 ? h.total - f0 : 0u;  // only rounds that hold a pair are looked up
      if (left > 192u) fused_select<4>(h, W, f0, lane, ws, js);
      else if (left > 128u) fused_select<3>(h, W, f0, lane, ws, js);
      else if (left > 64u) fused_select<2>(h, W, f0, lane, ws, js);
      else if (left > 0u) fused_select<1>(h, W, f0, lane, ws, js);
    };
    // requests a batch of pairs; nothing here waits for what it asks for (one tensor; with several,
    // the search for the pair's tensor does)
    auto fetch = [&](const FusedTile& h, uint32_t f0, FusedRaw<I> (&raw)[R]) {
      int ws[R];
      uint32_t js[R];
      select(h, f0, ws, js);
#pragma unroll
      for (int i = 0; i < R; ++i) {
        const uint32_t f = f0 + (uint32_t)(i * 64 + lane);
        raw[i].gi = (I)0;
        raw[i].sc = 0.0f;
        raw[i].qb = 0u;
        raw[i].aux = kNoPair;
        if (f < h.total) {
          const FusedWorker wk = s_wk[ws[i]];
          const uint32_t j = js[i];
          if (j < wk.k) {  // always, for lists that keep the contract
            raw[i].gi = static_cast<const I*>(wk.idx)[j];
            uint32_t rel_j = j;  // pair inside its tensor; sbase, qbase: the tensor's first scale and code byte
            long long sbase = 0, qbase = 0;
            if (T > 1) {  // blocks restart at every tensor: find the tensor that owns pair j
              int tl = 0, th = T - 1;
              if (T <= kFusedLdsTensors) {  // the tables are in LDS (every entry is below 2^32)
                while (tl < th) {
                  const int mid = (tl + th + 1) >> 1;
                  if (s_tp[0][mid] <= j) tl = mid; else th = mid - 1;
                }
                rel_j = j - s_tp[0][tl];
                sbase = (long long)s_tp[1][tl];
                qbase = (long long)s_tp[2][tl];
              } else {
                while (tl < th) {
                  const int mid = (tl + th + 1) >> 1;
                  if (kprefix[mid] <= (long long)j) tl = mid; else th = mid - 1;
                }
                rel_j = (uint32_t)((long long)j - kprefix[tl]);
                sbase = sprefix[tl];
                qbase = qprefix[tl];
              }
            }
            const uint32_t blk = fast_div(rel_j, bdiv);
            raw[i].sc = wk.sc[sbase + blk];
            if (codec == 0) {
              raw[i].qb = (uint32_t)(uint8_t)wk.q[qbase + rel_j];
              raw[i].aux = (uint32_t)ws[i] << 16;
            } else {  // sign code (Eq. 10): bit number rel_j - blk * block of the block's bytes
              const uint32_t bit = rel_j - blk * (uint32_t)block;
              raw[i].qb = (uint32_t)(uint8_t)wk.q[qbase + (long long)blk * sign_bytes + (bit >> 3)];
              raw[i].aux = ((uint32_t)ws[i] << 16) | (bit & 7u);
            }
          }
        }
      }
    };
    // value and position of a fetched pair, as a record of k_dec_tiles
    auto decode = [&](const FusedRaw<I>& p, int64_t base) -> uint2 {
      if (p.aux == kNoPair) return make_uint2(kNoRecord, 0u);
      const uint32_t w = p.aux >> 16;
      float val;
      if (codec == 0) val = __fmul_rn((float)(int8_t)(uint8_t)p.qb, p.sc);
      else val = ((p.qb >> (p.aux & 7u)) & 1u) ? p.sc : -p.sc;
      if (weighted) val = __fdiv_rn(val, s_wk[w].denom);  // Eq. 12: a stale worker counts for less
      const unsigned long long gi = (unsigned long long)p.gi, rel = gi - (unsigned long long)base;
      const uint32_t pos = (gi >= (unsigned long long)base && rel < (unsigned long long)kFusedTile) ? (uint32_t)rel : 0xFFFFu;
      return make_uint2(pos | (w << 16), __float_as_uint(val));
    };

    // sums one tile whose first batch of pairs has been requested, and writes it
    auto finish_tile = [&](const FusedTile& hc, FusedRaw<I> (&rc)[R], int ltile) {
      const int64_t base = (t0 + ltile) << tshift;
      const uint32_t total = hc.total;
      if (!(MODE == 1 && total == 0u)) {  // nothing to apply in an empty tile
        const f32x4 z = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int i = 0; i < kFusedTile / 256; ++i) *reinterpret_cast<f32x4*>(lt + (i * 64 + lane) * 4) = z;
        wave_sync();
#pragma unroll
        for (int i = 0; i < R; ++i) add_round<kFusedTile>(decode(rc[i], base), lt);
        for (uint32_t f0 = 64 * R; f0 < total; f0 += 64 * R) {  // a crowded tile: the rest, batch by batch
          FusedRaw<I> rx[R];
          fetch(hc, f0, rx);
#pragma unroll
          for (int i = 0; i < R; ++i) add_round<kFusedTile>(decode(rx[i], base), lt);
        }
        wave_sync();

        const int64_t remain = n - base;
        if (MODE == 0) {
          if (remain >= kFusedTile && ((reinterpret_cast<uintptr_t>(out) & 15u) == 0)) {
#pragma unroll
            for (int i = 0; i < kFusedTile / 256; ++i) {
              const f32x4 v = *reinterpret_cast<const f32x4*>(lt + (i * 64 + lane) * 4);
              __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(out + base + (i * 64 + lane) * 4));
            }
          } else {
            const int lim = (int)(remain < kFusedTile ? remain : kFusedTile);
            for (int i = lane; i < lim; i += 64) out[base + i] = lt[i];
          }
        } else {
          // every named position is claimed once (LDS exchange with a marker) and updated in place:
          // theta - fl32(c * sum). The positions are read again from the workers' lists (the lines were
          // fetched a moment ago); the loads of a batch of rounds are issued before its first store.
          for (uint32_t f0 = 0; f0 < total; f0 += 64 * R) {
            int ws[R];
            uint32_t js[R];
            select(hc, f0, ws, js);
            int64_t gi[R];
            float sum[R], th[R];
            bool mine[R];
#pragma unroll
            for (int i = 0; i < R; ++i) {
              const uint32_t f = f0 + (uint32_t)(i * 64 + lane);
              mine[i] = false;
              gi[i] = 0;
              sum[i] = 0.0f;
              if (f < total && js[i] < s_wk[ws[i]].k) {
                const unsigned long long g = (unsigned long long)static_cast<const I*>(s_wk[ws[i]].idx)[js[i]];
                const unsigned long long rel = g - (unsigned long long)base;
                if (g >= (unsigned long long)base && rel < (unsigned long long)kFusedTile && (int64_t)g < n) {
                  const uint32_t old = atomicExch(reinterpret_cast<uint32_t*>(lt) + (uint32_t)rel, kClaimed);
                  mine[i] = old != kClaimed;
                  sum[i] = __uint_as_float(old);
                  gi[i] = (int64_t)g;
                }
              }
            }
#pragma unroll
            for (int i = 0; i < R; ++i) th[i] = mine[i] ? out[gi[i]] : 0.0f;
#pragma unroll
            for (int i = 0; i < R; ++i)
              if (mine[i]) out[gi[i]] = __fsub_rn(th[i], __fmul_rn(c_apply, sum[i]));
          }
        }
        wave_sync();
      }
    };
    // Two sets of registers take turns: while one tile is summed out of one set, the next tile's
    // pairs arrive in the other (a copy between the sets would have to wait for them).
    FusedTile ha, hb;
    FusedRaw<I> ra[R], rb[R];
    // The first tile of a wavefront is its own number; after that it takes whichever tile of the
    // range is next (a counter in LDS), so that the wavefronts reach the end of the range together
    // whatever their tiles hold.
    int lt_cur = wave;
    auto tile_ok = [&](int ltile) { return ltile < tb && t0 + ltile < ntiles; };
    auto take_tile = [&]() {
      int v = 0;
      if (lane == 0) v = atomicAdd(s_next, 1);
      return __builtin_amdgcn_readfirstlane(v);
    };
    if (tile_ok(lt_cur)) {
      open_tile(lt_cur, ha);
      fetch(ha, 0u, ra);
      while (true) {
        int lt_next = take_tile();
        bool more = tile_ok(lt_next);
        if (more) {
          open_tile(lt_next, hb);
          fetch(hb, 0u, rb);
        }
        finish_tile(ha, ra, lt_cur);
        if (!more) break;
        lt_cur = lt_next;
        lt_next = take_tile();
        more = tile_ok(lt_next);
        if (more) {
          open_tile(lt_next, ha);
          fetch(ha, 0u, ra);
        }
        finish_tile(hb, rb, lt_cur);
        if (!more) break;
        lt_cur = lt_next;
      }
    }
  };

  if (PROD) {
    const bool prepares = wave >= kFusedWaves;
    int64_t r = blockIdx.x;
    int cur = 0;
    if (prepares && r < nranges) build(r, s_dyn, &s_next_tile[0]);
    __syncthreads();
    for (; r < nranges; r += gridDim.x, cur ^= 1) {
      const int64_t rn = r + gridDim.x;
      if (prepares) {
        if (rn < nranges) build(rn, s_dyn + (cur ^ 1) * tab_len, &s_next_tile[cur ^ 1]);
      } else {
        consume(r, s_dyn + cur * tab_len, &s_next_tile[cur]);
      }
      __syncthreads();  // the next range's table is complete, and this one's may be rewritten
    }
  } else {
    for (int64_t r = blockIdx.x; r < nranges; r += gridDim.x) {
      build(r, s_dyn, &s_next_tile[0]);
      consume(r, s_dyn, &s_next_tile[0]);
      __syncthreads();  // the table is rewritten for the next range
    }
  }
}

// All wavefronts prepare and take tiles (WAVES / 2 wavefronts per SIMD: two workgroups per compute unit).
template <typename I, int MODE, int TSHIFT, int WAVES>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(WAVES / 2, WAVES / 2))) void k_dec_fused(
    DecArgs a, int W, int tb, int32_t block, FastDiv bdiv, int64_t ntiles, int64_t nranges, int codec, int weighted,
    int64_t n, const long long* __restrict__ kprefix, const long long* __restrict__ sprefix,
    const long long* __restrict__ qprefix, int T, float* __restrict__ out, float c_apply) {
  dec_fused_body<I, MODE, TSHIFT, WAVES, 0>(a, W, tb, block, bdiv, ntiles, nranges, codec, weighted, n, kprefix, sprefix,
                                            qprefix, T, out, c_apply);
}

// With PROD preparing wavefronts: one workgroup per compute unit (its tiles take most of the LDS).
template <typename I, int MODE, int TSHIFT, int WAVES, int PROD>
__global__ __launch_bounds__((WAVES + PROD) * 64) void k_dec_fused_prep(
    DecArgs a, int W, int tb, int32_t block, FastDiv bdiv, int64_t ntiles, int64_t nranges, int codec, int weighted,
    int64_t n, const long long* __restrict__ kprefix, const long long* __restrict__ sprefix,
    const long long* __restrict__ qprefix, int T, float* __restrict__ out, float c_apply) {
  dec_fused_body<I, MODE, TSHIFT, WAVES, PROD>(a, W, tb, block, bdiv, ntiles, nranges, codec, weighted, n, kprefix,
                                               sprefix, qprefix, T, out, c_apply);
}

}  // namespace

// log2 of the tile size for a call: large tiles for long, thinly filled vectors.
int dec_tile_shift(int64_t nrec, int64_t n) {
  const double per_small = (double)nrec * (1 << kDecTileShiftSmall) / (double)(n > 0 ? n : 1);
  return (n >= (int64_t(1) << 28) && per_small <= 96.0) ? kDecTileShiftLarge : kDecTileShiftSmall;
}

int dec_tile_shift_of(bool large) { return large ? kDecTileShiftLarge : kDecTileShiftSmall; }

// Tiles per range of the packing pass: as many as make a range 2^19 output floats (128 small
// tiles; half that with many workers: the LDS tables hold (2 * tiles + 1) * W entries), fewer when
// the tiles are crowded or the vector is short, so that a range stays a small piece of work and
// there are enough ranges to fill the chip. A power of two, at least 8.
int dec_range_tiles(int W, int tshift, int64_t nrec, int64_t n) {
  const double per_tile = (double)nrec * (double)(int64_t(1) << tshift) / (double)(n > 0 ? n : 1);
  const int64_t ntiles = (n + (int64_t(1) << tshift) - 1) >> tshift;
  int tb = (W <= 32 ? (1 << 19) : (1 << 18)) >> tshift;
  while (tb > 8 && (per_tile * tb > 32768.0 || ntiles / tb < 2048)) tb >>= 1;
  return tb;
}

// Tiles per range of the fused kernel: the LDS table holds (tb + 1) * W entries (about 8 KB), and
// there should be enough ranges to keep two workgroups per compute unit busy. A power of two >= 4.
int dec_fused_range_tiles(int W, int64_t n, int tshift, int tables) {
  const int64_t ntiles = (n + (int64_t(1) << tshift) - 1) >> tshift;
  int tb = 128;
  while (tb > 4 && ((tb + 1) * W > 2112 || ntiles / tb < 1024)) tb >>= 1;
  return tb;
}

template <int TSHIFT, int WAVES, int PROD>
static void launch_fused_shape(const DecArgs& a, int W, int index_bits, int32_t block, int codec, int weighted, int64_t n,
                               const long long* kprefix, const long long* sprefix, const long long* qprefix, int T,
                               float* out, int apply, float c_apply, hipStream_t s) {
  const int tb = dec_fused_range_tiles(W, n, TSHIFT, PROD ? 2 : 1);
  const int64_t ntiles = (n + (int64_t(1) << TSHIFT) - 1) >> TSHIFT;
  const int64_t nranges = (ntiles + tb - 1) / tb;
  const int64_t wgs = PROD ? 256 : 512;  // one workgroup per compute unit with preparing wavefronts, else two
  const dim3 grid((unsigned)(nranges < wgs ? nranges : wgs)), blk((WAVES + PROD) * 64);
  const size_t lds = sizeof(uint32_t) * (size_t)(tb + 1) * W * (PROD ? 2 : 1);
  const FastDiv bdiv = make_fastdiv((uint32_t)block);
#define GC_LAUNCH_FUSED(ITYPE, MODE)                                                                                 \
  do {                                                                                                               \
    if constexpr (PROD != 0)                                                                                         \
      hipLaunchKernelGGL((k_dec_fused_prep<ITYPE, MODE, TSHIFT, WAVES, PROD>), grid, blk, lds, s, a, W, tb,            \
                         block, bdiv, ntiles, nranges, codec, weighted, n, kprefix, sprefix, qprefix, T, out, c_apply); \
    else                                                                                                             \
      hipLaunchKernelGGL((k_dec_fused<ITYPE, MODE, TSHIFT, WAVES>), grid, blk, lds, s, a, W, tb, block, bdiv, ntiles,  \
                         nranges, codec, weighted, n, kprefix, sprefix, qprefix, T, out, c_apply);                    \
  } while (0)
  if (index_bits == 32) {
    if (apply) GC_LAUNCH_FUSED(uint32_t, 1); else GC_LAUNCH_FUSED(uint32_t, 0);
  } else {
    if (apply) GC_LAUNCH_FUSED(unsigned long long, 1); else GC_LAUNCH_FUSED(unsigned long long, 0);
  }
#undef GC_LAUNCH_FUSED
}

void launch_dec_fused(const DecArgs& a, int W, int index_bits, int32_t block, int codec, int weighted, int64_t n,
                      const long long* kprefix, const long long* sprefix, const long long* qprefix, int T, float* out,
                      int apply, float c_apply, int crowded, hipStream_t s) {
  if (crowded)
    launch_fused_shape<kFusedTileShift, kFusedWavesCrowded, 0>(a, W, index_bits, block, codec, weighted, n, kprefix, sprefix,
                                                               qprefix, T, out, apply, c_apply, s);
  else
    launch_fused_shape<kFusedTileShift, kFusedWavesThin, kFusedPrepThin>(a, W, index_bits, block, codec, weighted, n, kprefix,
                                                                         sprefix, qprefix, T, out, apply, c_apply, s);
}

void launch_dec_pack(const DecArgs& a, int W, int index_bits, int tb, int tshift, int32_t block, int64_t ntiles,
                     int64_t r_first, int64_t r_count, const long long* kprefix, const long long* sprefix,
                     const long long* qprefix, int T, int codec, int weighted, void* rec, unsigned long long* tile_start,
                     hipStream_t s) {
  const dim3 grid((unsigned)r_count);
  const size_t lds = sizeof(uint32_t) * (size_t)(2 * tb + 1) * W;  // at most 33 KB
  const FastDiv bdiv = make_fastdiv((uint32_t)block);
  if (index_bits == 32)
    hipLaunchKernelGGL(k_dec_pack<uint32_t>, grid, dim3(kPackThreads), lds, s, a, W, tb, tshift, block, bdiv, ntiles, r_first,
                       kprefix, sprefix, qprefix, T, codec, weighted, (uint2*)rec, tile_start);
  else
    hipLaunchKernelGGL(k_dec_pack<unsigned long long>, grid, dim3(kPackThreads), lds, s, a, W, tb, tshift, block, bdiv, ntiles,
                       r_first, kprefix, sprefix, qprefix, T, codec, weighted, (uint2*)rec, tile_start);
}

template <int TSHIFT, int WAVES>
static void launch_tiles_shape(const void* rec, const unsigned long long* tile_start, uint64_t nrec, int64_t n,
                               int64_t t_begin, int64_t t_end, float* out, int apply, float c_apply,
                               unsigned apply_dense_min, hipStream_t s) {
  const int64_t want = (t_end - t_begin + WAVES - 1) / WAVES;
  const dim3 grid((unsigned)(want < kDecGrid ? want : kDecGrid)), blk(WAVES * 64);
  if (apply)
    hipLaunchKernelGGL((k_dec_tiles<1, (1 << TSHIFT), WAVES>), grid, blk, 0, s, (const uint2*)rec, tile_start,
                       (unsigned long long)nrec, n, t_begin, t_end, out, c_apply, apply_dense_min);
  else
    hipLaunchKernelGGL((k_dec_tiles<0, (1 << TSHIFT), WAVES>), grid, blk, 0, s, (const uint2*)rec, tile_start,
                       (unsigned long long)nrec, n, t_begin, t_end, out, c_apply, apply_dense_min);
}

void launch_dec_tiles(const void* rec, const unsigned long long* tile_start, uint64_t nrec, int tshift, int64_t n,
                      int64_t t_begin, int64_t t_end, float* out, int apply, float c_apply, unsigned apply_dense_min,
                      hipStream_t s) {
  if (t_end <= t_begin) return;
  // apply_dense_min counts records per 4096 floats; a large tile holds four times as many
  if (tshift == kDecTileShiftLarge)
    launch_tiles_shape<kDecTileShiftLarge, kDecWavesLarge>(rec, tile_start, nrec, n, t_begin, t_end, out, apply, c_apply,
                                                            apply_dense_min << (kDecTileShiftLarge - kDecTileShiftSmall), s);
  else
    launch_tiles_shape<kDecTileShiftSmall, kDecWavesSmall>(rec, tile_start, nrec, n, t_begin, t_end, out, apply, c_apply,
                                                            apply_dense_min, s);
}

}  // namespace gc
