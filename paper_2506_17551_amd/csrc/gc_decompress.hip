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

typedef float f32x4 __attribute__((ext_vector_type(4)));

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

template <typename I>
__global__ __launch_bounds__(kDecWaves * 64) void k_dec_tiles(DecArgs a, int W, int32_t block, int64_t n,
                                                   int64_t ntiles, const uint32_t* __restrict__ bounds,
                                                   const long long* __restrict__ kprefix,
                                                   const long long* __restrict__ sprefix, int T,
                                                   float* __restrict__ out) {
  __shared__ float tile_mem[kDecWaves][kDecTile];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float* lt = tile_mem[wave];
  // wavefronts walk the tiles with a grid stride; no workgroup barrier is used in the loop
  for (int64_t tile = (int64_t)blockIdx.x * kDecWaves + wave; tile < ntiles;
       tile += (int64_t)gridDim.x * kDecWaves) {
  const int64_t base = tile * kDecTile;
  const f32x4 z = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int i = 0; i < kDecTile / 256; ++i) *reinterpret_cast<f32x4*>(lt + (i * 64 + lane) * 4) = z;

  // lane w holds worker w's pair range for this tile
  uint32_t lo = 0, cnt = 0;
  if (lane < W) {
    lo = bounds[tile * W + lane];
    cnt = bounds[(tile + 1) * W + lane] - lo;
  }
  uint32_t incl = cnt;  // inclusive scan over lanes
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t u = __shfl_up(incl, off);
    if (lane >= off) incl += u;
  }
  const uint32_t total = __shfl(incl, 63);
  const uint32_t excl = incl - cnt;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();

  for (uint32_t s0 = 0; s0 < total; s0 += 64) {
    const uint32_t sidx = s0 + lane;
    const bool active = sidx < total;
    // owner worker of slot sidx: the last w with excl[w] <= sidx among workers that have pairs
    int myw = 0;
    uint32_t myj = 0;
    for (int w = 0; w < W; ++w) {  // w is wave-uniform: scalar lane reads
      const uint32_t ex = (uint32_t)__builtin_amdgcn_readlane((int)excl, w);
      const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)cnt, w);
      const uint32_t l = (uint32_t)__builtin_amdgcn_readlane((int)lo, w);
      if (c != 0u && sidx >= ex) { myw = w; myj = l + (sidx - ex); }
    }
    float val = 0.0f;
    uint32_t pos = 0;
    if (active) {
      const I* idx = static_cast<const I*>(a.indices[myw]);
      pos = (uint32_t)((unsigned long long)idx[myj] - (unsigned long long)base);
      const int code = a.q[myw][myj];
      long long sj = (long long)myj / block;
      if (T > 1) {  // scales restart at every tensor: find the tensor that owns pair myj
        int tl = 0, th = T - 1;
        while (tl < th) {
          const int mid = (tl + th + 1) >> 1;
          if (kprefix[mid] <= (long long)myj) tl = mid; else th = mid - 1;
        }
        sj = sprefix[tl] + ((long long)myj - kprefix[tl]) / block;
      }
      val = __fmul_rn((float)code, a.scales[myw][sj]);
    }
    // add worker by worker so that equal indices of different workers keep ascending order
    const uint64_t act = __ballot(active);
    const int w_first = __shfl(myw, __ffsll((unsigned long long)act) - 1);
    const int w_last = __shfl(myw, 63 - __clzll((unsigned long long)act));
    for (int w = w_first; w <= w_last; ++w) {
      if (active && myw == w && pos < (uint32_t)kDecTile) lt[pos] = __fadd_rn(lt[pos], val);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }

  const int64_t remain = n - base;
  if (remain >= kDecTile && ((reinterpret_cast<uintptr_t>(out) & 15u) == 0)) {
#pragma unroll
    for (int i = 0; i < kDecTile / 256; ++i) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(lt + (i * 64 + lane) * 4);
#if defined(GC_DEC_PLAIN_STORE)
      *reinterpret_cast<f32x4*>(out + base + (i * 64 + lane) * 4) = v;
#else
      __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(out + base + (i * 64 + lane) * 4));
#endif
    }
  } else {
    const int lim = (int)(remain < kDecTile ? remain : kDecTile);
    for (int i = lane; i < lim; i += 64) out[base + i] = lt[i];
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  }  // tile loop
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
                      const uint32_t* bounds, const long long* kprefix, const long long* sprefix, int T,
                      float* out, hipStream_t s) {
#ifndef GC_DEC_GRID
#define GC_DEC_GRID 512
#endif
#if GC_DEC_GRID > 0
  const int64_t want = (ntiles + kDecWaves - 1) / kDecWaves;
  const dim3 grid((unsigned)(want < GC_DEC_GRID ? want : GC_DEC_GRID));
#else
  const dim3 grid((unsigned)((ntiles + kDecWaves - 1) / kDecWaves));
#endif
  if (index_bits == 32)
    hipLaunchKernelGGL(k_dec_tiles<uint32_t>, grid, dim3(kDecWaves * 64), 0, s, a, W, block, n, ntiles, bounds,
                       kprefix, sprefix, T, out);
  else
    hipLaunchKernelGGL(k_dec_tiles<unsigned long long>, grid, dim3(kDecWaves * 64), 0, s, a, W, block, n, ntiles,
                       bounds, kprefix, sprefix, T, out);
}

}  // namespace gc
