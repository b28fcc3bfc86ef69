// Decompress-and-sum: the aggregate of W workers' compressed gradients as a dense
// fp32 vector (paper Sec. III.B, Eq. 8 without the 1/P), for gfx950.
//
//   k_dec_bounds  for every worker and every output tile, the first pair whose index falls
//                 in the tile (binary search in the worker's ascending index list).
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
__global__ __launch_bounds__(256) void k_dec_bounds(DecArgs a, int W, int64_t ntiles,
                                                    uint32_t* __restrict__ bounds) {
  const int64_t per = ntiles + 1;
  const int64_t total = per * W;
  for (int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; id < total;
       id += (int64_t)gridDim.x * blockDim.x) {
    const int w = (int)(id / per);
    const int64_t tile = id - (int64_t)w * per;
    const I* idx = static_cast<const I*>(a.indices[w]);
    const unsigned long long target = (unsigned long long)tile * kDecTile;
    uint32_t lo = 0, hi = a.k[w];  // first j in [0, k] with idx[j] >= target
    while (lo < hi) {
      const uint32_t mid = lo + ((hi - lo) >> 1);
      if ((unsigned long long)idx[mid] < target) lo = mid + 1; else hi = mid;
    }
    bounds[id] = lo;
  }
}

template <typename I>
__global__ __launch_bounds__(256) void k_dec_tiles(DecArgs a, int W, int32_t block, int64_t n,
                                                   int64_t ntiles, const uint32_t* __restrict__ bounds,
                                                   const long long* __restrict__ kprefix,
                                                   const long long* __restrict__ sprefix, int T,
                                                   float* __restrict__ out) {
  __shared__ float tile_mem[4][kDecTile];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t tile = (int64_t)blockIdx.x * 4 + wave;
  if (tile >= ntiles) return;  // no workgroup barrier is used below
  float* lt = tile_mem[wave];
  const int64_t base = tile * kDecTile;
  const f32x4 z = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int i = 0; i < kDecTile / 256; ++i) *reinterpret_cast<f32x4*>(lt + (i * 64 + lane) * 4) = z;

  // lane w holds worker w's pair range for this tile
  uint32_t lo = 0, cnt = 0;
  if (lane < W) {
    lo = bounds[(int64_t)lane * (ntiles + 1) + tile];
    cnt = bounds[(int64_t)lane * (ntiles + 1) + tile + 1] - lo;
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
      __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(out + base + (i * 64 + lane) * 4));
    }
  } else {
    const int lim = (int)(remain < kDecTile ? remain : kDecTile);
    for (int i = lane; i < lim; i += 64) out[base + i] = lt[i];
  }
}

}  // namespace

void launch_dec_bounds(const DecArgs& a, int W, int index_bits, int64_t ntiles, uint32_t* bounds,
                       hipStream_t s) {
  const int64_t total = (ntiles + 1) * W;
  int64_t blocks = (total + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  if (index_bits == 32)
    hipLaunchKernelGGL(k_dec_bounds<uint32_t>, dim3((unsigned)blocks), dim3(256), 0, s, a, W, ntiles, bounds);
  else
    hipLaunchKernelGGL(k_dec_bounds<unsigned long long>, dim3((unsigned)blocks), dim3(256), 0, s, a, W,
                       ntiles, bounds);
}

void launch_dec_tiles(const DecArgs& a, int W, int index_bits, int32_t block, int64_t n, int64_t ntiles,
                      const uint32_t* bounds, const long long* kprefix, const long long* sprefix, int T,
                      float* out, hipStream_t s) {
  const dim3 grid((unsigned)((ntiles + 3) / 4));
  if (index_bits == 32)
    hipLaunchKernelGGL(k_dec_tiles<uint32_t>, grid, dim3(256), 0, s, a, W, block, n, ntiles, bounds,
                       kprefix, sprefix, T, out);
  else
    hipLaunchKernelGGL(k_dec_tiles<unsigned long long>, grid, dim3(256), 0, s, a, W, block, n, ntiles,
                       bounds, kprefix, sprefix, T, out);
}

}  // namespace gc
