// Decompress-and-sum: the aggregate of W workers' compressed gradients as a dense
// fp32 vector (paper Sec. III.B, Eq. 8 without the 1/P), for gfx950.
//
//   k_dec_bounds  for every output tile and every worker, the first pair whose index falls
//                 in the tile (bracketed binary search in the worker's ascending index list).
//   k_dec_tiles   one wavefront per tile of kDecTile output floats held in LDS: the pairs of
//                 all workers that fall in the tile are decoded in parallel across lanes and
//                 added into the LDS tile worker by worker (ascending), then the tile is
//                 written out once with 128-bit stores. Every output byte is written exactly
//                 once; there is no separate memset and no global atomic. Because indices are
//                 unique inside one worker's buffer, the adds of one worker never collide, and
//                 the fixed worker order makes the fp32 sum reproducible bit for bit.
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

// bounds[tile * W + w] = first pair of worker w whose index is >= tile * kDecTile, for tile in
// [0, ntiles]. A workgroup covers 256 consecutive tiles of all workers: 2W lanes bracket the
// workgroup's range with full binary searches, then every (tile, worker) is searched inside its
// worker's bracket (a few hundred pairs that stay in cache). Consecutive threads write
// consecutive entries, so the table leaves the chip as whole lines.
template <typename I>
__global__ __launch_bounds__(256) void k_dec_bounds(DecArgs a, int W, int64_t ntiles,
                                                    uint32_t* __restrict__ bounds) {
  __shared__ uint32_t s_br[2][kMaxWorkers];
  const int64_t t0 = (int64_t)blockIdx.x * 256;
  if ((int)threadIdx.x < 2 * W) {
    const int w = threadIdx.x % W, side = threadIdx.x / W;
    s_br[side][w] = lower_bound_idx<I>(static_cast<const I*>(a.indices[w]), 0u, a.k[w],
                                       (unsigned long long)(t0 + 256 * side) * kDecTile);
  }
  __syncthreads();
  for (int flat = threadIdx.x; flat < 256 * W; flat += 256) {
    const int w = flat % W;
    const int64_t tile = t0 + flat / W;
    if (tile > ntiles) break;
    bounds[tile * W + w] = lower_bound_idx<I>(static_cast<const I*>(a.indices[w]), s_br[0][w], s_br[1][w],
                                              (unsigned long long)tile * kDecTile);
  }
}

#ifndef GC_DEC_WAVES
#define GC_DEC_WAVES 8
#endif
constexpr int kDecWaves = GC_DEC_WAVES;  // wavefronts (= tiles) per workgroup
#ifndef GC_DEC_GRID
#define GC_DEC_GRID 512
#endif
constexpr int kDecGrid = GC_DEC_GRID;    // persistent workgroups (2 per CU)

// What one lane decodes in one round of a tile: a pair of some worker, or nothing.
struct LanePair {
  bool active;
  int w;         // worker
  uint32_t j;    // pair index in that worker's buffer
};

// Pair number (s0 + lane) of the tile, counting the workers' pairs in worker order.
__device__ __forceinline__ LanePair locate_pair(uint32_t s0, int lane, uint32_t total, int W, uint32_t excl,
                                                uint32_t cnt, uint32_t lo) {
  LanePair p;
  const uint32_t sidx = s0 + lane;
  p.active = sidx < total;
  p.w = 0;
  p.j = 0;
  for (int w = 0; w < W; ++w) {  // w is wave-uniform: scalar lane reads
    const uint32_t ex = (uint32_t)__builtin_amdgcn_readlane((int)excl, w);
    const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)cnt, w);
    const uint32_t l = (uint32_t)__builtin_amdgcn_readlane((int)lo, w);
    if (c != 0u && sidx >= ex) { p.w = w; p.j = l + (sidx - ex); }
  }
  return p;
}

constexpr uint32_t kClaimed = 0x7FC0DEADu;  // a NaN pattern no finite sum can produce

// The pair range of every worker inside one tile: lane w holds worker w's first pair and count,
// `excl` the number of pairs of the workers before it, `total` the tile's pairs over all workers.
struct TileBounds {
  uint32_t lo, cnt, excl, total;
};

__device__ __forceinline__ void load_bounds(const uint32_t* __restrict__ bounds, int64_t tile, int W, int lane,
                                            uint32_t& lo, uint32_t& hi) {
  lo = 0u;
  hi = 0u;
  if (lane < W) {
    lo = bounds[tile * W + lane];
    hi = bounds[(tile + 1) * W + lane];
  }
}

__device__ __forceinline__ TileBounds scan_bounds(uint32_t lo, uint32_t hi, int lane) {
  TileBounds b;
  b.lo = lo;
  // every bound lies in [0, k], so a pair number below lo + cnt is always a valid one; unsorted
  // indices (which break the caller's contract) can only make hi < lo, and then the tile is skipped
  b.cnt = hi > lo ? hi - lo : 0u;
  uint32_t incl = b.cnt;  // inclusive scan over lanes
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t u = __shfl_up(incl, off);
    if (lane >= off) incl += u;
  }
  b.total = __shfl(incl, 63);
  b.excl = incl - b.cnt;
  return b;
}

// The pair a lane decodes in one round, as loaded: index, scale and raw code.
struct PairLoad {
  LanePair p;
  unsigned long long gi;  // index in the dense vector
  float s;                // scale of the pair's block
  uint32_t code;          // int8 code (low byte), or the sign byte << 8 | bit number
};

// Issues the loads of round s0 of a tile together; nothing here consumes their results, so the
// index, scale and code of a pair cost one round trip to memory, not three.
template <typename I>
__device__ __forceinline__ PairLoad load_pairs(const DecArgs& a, uint32_t s0, int lane, int W, const TileBounds& b,
                                              int32_t block, const long long* __restrict__ kprefix,
                                              const long long* __restrict__ sprefix,
                                              const long long* __restrict__ qprefix, int T, int codec) {
  PairLoad c;
  c.p = locate_pair(s0, lane, b.total, W, b.excl, b.cnt, b.lo);
  c.gi = 0ull;
  c.s = 0.0f;
  c.code = 0u;
  if (c.p.active) {
    const I* idx = static_cast<const I*>(a.indices[c.p.w]);
    const float* sc = a.scales[c.p.w];
    const int8_t* qw = a.q[c.p.w];
    c.gi = (unsigned long long)idx[c.p.j];
    long long rel = (long long)c.p.j, sbase = 0, qbase = 0;  // pair inside its tensor; tensor's scales, bytes
    if (T > 1) {  // blocks restart at every tensor: find the tensor that owns pair j
      int tl = 0, th = T - 1;
      while (tl < th) {
        const int mid = (tl + th + 1) >> 1;
        if (kprefix[mid] <= (long long)c.p.j) tl = mid; else th = mid - 1;
      }
      rel -= kprefix[tl];
      sbase = sprefix[tl];
      qbase = qprefix[tl];
    }
    const long long blk = rel / block;
    c.s = sc[sbase + blk];
    if (codec == 0) {
      c.code = (uint8_t)qw[T > 1 ? qbase + rel : rel];
    } else {  // sign code (Eq. 10): bit r of the block's bytes
      c.code = (uint32_t)(rel - blk * block);  // r; the byte is loaded below, the bit taken at use
      c.code = (c.code & 7u) | ((uint32_t)(uint8_t)qw[qbase + blk * ((block + 7) / 8) + (c.code >> 3)] << 8);
    }
  }
  return c;
}

__device__ __forceinline__ void wave_sync() {  // orders the wavefront's own LDS accesses
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// Adds one round of pairs into the wavefront's LDS tile so that equal indices of different workers
// are added in ascending worker order: one LDS float add (round to nearest even, denormals kept,
// like the plain fp32 add) per worker present in the round, issued back to back. The LDS executes
// a wavefront's instructions in the order they were issued, so nothing has to wait in between, and
// within one worker the indices are unique, so the lanes of one instruction never collide.
__device__ __forceinline__ void add_pairs(const DecArgs& a, const PairLoad& c, int64_t base, int codec,
                                          int weighted, float* lt) {
  float val = 0.0f;
  uint32_t pos = 0xFFFFFFFFu;
  if (c.p.active) {
    pos = (uint32_t)(c.gi - (unsigned long long)base);
    if (codec == 0) val = __fmul_rn((float)(int8_t)c.code, c.s);
    else val = ((c.code >> (8 + (c.code & 7u))) & 1u) ? c.s : -c.s;
    if (weighted) val = __fdiv_rn(val, a.denom[c.p.w]);  // Eq. 12: a stale worker counts for less
  }
  const bool act = c.p.active && pos < (uint32_t)kDecTile;
  const uint64_t am = __ballot(act);
  if (am == 0ull) return;
  const int w_first = __shfl(c.p.w, __ffsll((unsigned long long)am) - 1);
  const int w_last = __shfl(c.p.w, 63 - __clzll((unsigned long long)am));
  for (int w = w_first; w <= w_last; ++w) {
    if (act && c.p.w == w) (void)__hip_atomic_fetch_add(lt + pos, val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
    __builtin_amdgcn_wave_barrier();  // keeps the instructions in this order
  }
  wave_sync();
}

// MODE 0: out[tile] = sum (dense write).  MODE 1: theta[i] -= c * sum[i] at the touched i only.
// Wavefronts walk the tiles with a grid stride, without workgroup barriers. Fetching a
// wavefront's next tile ahead of time (its bounds, or its pairs) measured slower on the 7B workload
// than this plain order, as did keeping the workers' pointers in LDS.
template <typename I, int MODE>
__global__ __launch_bounds__(kDecWaves * 64) void k_dec_tiles(DecArgs a, int W, int32_t block, int64_t n,
                                                   int64_t ntiles, const uint32_t* __restrict__ bounds,
                                                   const long long* __restrict__ kprefix,
                                                   const long long* __restrict__ sprefix,
                                                   const long long* __restrict__ qprefix, int T, int codec,
                                                   float* __restrict__ out, int weighted, float c_apply) {
  __shared__ float tile_mem[kDecWaves][kDecTile];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float* lt = tile_mem[wave];
  const int64_t stride = (int64_t)gridDim.x * kDecWaves;
  int64_t tile = (int64_t)blockIdx.x * kDecWaves + wave;
  if (tile >= ntiles) return;

  for (; tile < ntiles; tile += stride) {
    const int64_t base = tile * kDecTile;
    uint32_t lo, hi;
    load_bounds(bounds, tile, W, lane, lo, hi);
    const TileBounds cur = scan_bounds(lo, hi, lane);

    if (!(MODE == 1 && cur.total == 0u)) {  // MODE 1: nothing to apply in an empty tile
      const f32x4 z = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int i = 0; i < kDecTile / 256; ++i) *reinterpret_cast<f32x4*>(lt + (i * 64 + lane) * 4) = z;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();

      const PairLoad first = load_pairs<I>(a, 0u, lane, W, cur, block, kprefix, sprefix, qprefix, T, codec);
      add_pairs(a, first, base, codec, weighted, lt);
      for (uint32_t s0 = 64; s0 < cur.total; s0 += 64) {
        const PairLoad c = load_pairs<I>(a, s0, lane, W, cur, block, kprefix, sprefix, qprefix, T, codec);
        add_pairs(a, c, base, codec, weighted, lt);
      }

      if (MODE == 0) {
        const int64_t remain = n - base;
        if (remain >= kDecTile && ((reinterpret_cast<uintptr_t>(out) & 15u) == 0)) {
#pragma unroll
          for (int i = 0; i < kDecTile / 256; ++i) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(lt + (i * 64 + lane) * 4);
            __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(out + base + (i * 64 + lane) * 4));
          }
        } else {
          const int lim = (int)(remain < kDecTile ? remain : kDecTile);
          for (int i = lane; i < lim; i += 64) out[base + i] = lt[i];
        }
      } else {
        // every touched position is claimed once (LDS exchange with a marker) and updated in place:
        // theta - fl32(c * sum). Untouched positions have sum +0 and would not change anyway.
        for (uint32_t s0 = 0; s0 < cur.total; s0 += 64) {
          const LanePair p = locate_pair(s0, lane, cur.total, W, cur.excl, cur.cnt, cur.lo);
          if (p.active) {
            const I* idx = static_cast<const I*>(a.indices[p.w]);
            const unsigned long long gi = (unsigned long long)idx[p.j];
            const uint32_t pos = (uint32_t)(gi - (unsigned long long)base);
            if (pos < (uint32_t)kDecTile && gi < (unsigned long long)n) {
              const uint32_t old = atomicExch(reinterpret_cast<uint32_t*>(lt) + pos, kClaimed);
              if (old != kClaimed) out[gi] = __fsub_rn(out[gi], __fmul_rn(c_apply, __uint_as_float(old)));
            }
          }
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }
}

}  // namespace

void launch_dec_bounds(const DecArgs& a, int W, int index_bits, int64_t ntiles, uint32_t* bounds,
                       hipStream_t s) {
  const dim3 grid((unsigned)((ntiles + 1 + 255) / 256));
  if (index_bits == 32)
    hipLaunchKernelGGL(k_dec_bounds<uint32_t>, grid, dim3(256), 0, s, a, W, ntiles, bounds);
  else
    hipLaunchKernelGGL(k_dec_bounds<unsigned long long>, grid, dim3(256), 0, s, a, W, ntiles, bounds);
}

void launch_dec_tiles(const DecArgs& a, int W, int index_bits, int32_t block, int64_t n, int64_t ntiles,
                      const uint32_t* bounds, const long long* kprefix, const long long* sprefix,
                      const long long* qprefix, int T, int codec, float* out, int weighted, int apply,
                      float c_apply, hipStream_t s) {
  const int64_t want = (ntiles + kDecWaves - 1) / kDecWaves;
  const dim3 grid((unsigned)(want < kDecGrid ? want : kDecGrid)), blk(kDecWaves * 64);
#define GC_LAUNCH_TILES(ITYPE, MODE)                                                                        \
  hipLaunchKernelGGL((k_dec_tiles<ITYPE, MODE>), grid, blk, 0, s, a, W, block, n, ntiles, bounds, kprefix, \
                     sprefix, qprefix, T, codec, out, weighted, c_apply)
  if (index_bits == 32) {
    if (apply) GC_LAUNCH_TILES(uint32_t, 1); else GC_LAUNCH_TILES(uint32_t, 0);
  } else {
    if (apply) GC_LAUNCH_TILES(unsigned long long, 1); else GC_LAUNCH_TILES(unsigned long long, 0);
  }
#undef GC_LAUNCH_TILES
}

}  // namespace gc
