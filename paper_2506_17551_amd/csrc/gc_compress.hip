// Compress side: error-feedback accumulate, exact magnitude top-k, per-block int8
// codes and the fused residual write-back (paper Sec. III.B, Eq. 11), for gfx950.
//
// Shape of the computation
//   The flat gradient is cut into ITEMS of item_len consecutive elements; one
//   wavefront owns one item, one workgroup owns kItemsPerGroup consecutive items of one tensor.
//   1. k_sample       reads a small slice of every item, forms acc = g + e there and
//                     histograms the top 13 key bits; k_sample_thresh turns that into a
//                     candidate threshold t_lo that, with overwhelming probability, is
//                     below the true k-th largest key.
//   2. k_main         the one full streaming pass: acc = g + e with 128-bit loads, acc
//                     written over e, and every entry with key >= t_lo appended, in
//                     ascending index order, to the item's candidate slots.
//   3. k_hist / k_select_scan (x3)  exact radix select of the k-th largest key T and the
//                     tie quota over the candidates (LDS histograms per workgroup).
//   4. k_count / k_item_scan / k_emit   ordered compaction (wavefront ballot + prefix) of
//                     the kept entries: key > T, or key == T among the first `quota` such.
//   5. k_quant        per block of kept entries: amax, scale, int8 codes, and the residual
//                     at the kept positions (acc - q*s).
//   Small or high-density tensors skip 1 and the candidate gathering: k_main histograms the
//   first digit itself and steps 3-4 read the dense residual (which then holds acc). A
//   sampled tensor whose candidates turn out to be too few (or overflow their slots) takes
//   the same dense route, so the result never depends on the sample.
#include "gc_internal.h"

namespace gc {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t mbcnt64(uint64_t m) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}
__device__ __forceinline__ uint32_t key_of(float x) { return __float_as_uint(x) & 0x7FFFFFFFu; }
__device__ __forceinline__ float bf16_widen(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

template <typename G> __device__ __forceinline__ float load_grad(const G* g, int64_t i);
template <> __device__ __forceinline__ float load_grad<float>(const float* g, int64_t i) { return g[i]; }
template <> __device__ __forceinline__ float load_grad<uint16_t>(const uint16_t* g, int64_t i) {
  return bf16_widen(g[i]);
}

// Largest t with td[t].item_begin <= item.
__device__ __forceinline__ int find_tensor_by_item(const TensorDesc* td, int T, int64_t item, int hint) {
  if (T == 1) return 0;
  if (item >= td[hint].item_begin && item < td[hint].item_end) return hint;
  int lo = 0, hi = T - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (td[mid].item_begin <= item) lo = mid; else hi = mid - 1;
  }
  return lo;
}

__device__ __forceinline__ bool fast_path_failed(const TensorState& st, const TensorDesc& d) {
  return st.overflow != 0u || st.cand_total < (unsigned long long)d.k;
}

// ---------------------------------------------------------------- k_init
__global__ __launch_bounds__(256) void k_init(Workspace ws) {
  const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t ns = (int64_t)ws.T * kSampleBins, nh = (int64_t)ws.T * kSelBins;
  for (int64_t i = tid; i < ns; i += stride) ws.shist[i] = 0ull;
  for (int64_t i = tid; i < nh; i += stride) ws.hist[i] = 0ull;
  for (int64_t i = tid; i < ws.T; i += stride) {
    TensorState z;
    z.cand_total = 0ull; z.k_rem = 0ull; z.t_lo = 0u; z.overflow = 0u; z.prefix = 0u; z.pad_ = 0u;
    ws.ts[i] = z;
  }
}

// ---------------------------------------------------------------- LDS histogram flush
template <int NB>
__device__ __forceinline__ void flush_lds_hist(uint32_t* lh, unsigned long long* gh) {
  for (int b = threadIdx.x; b < NB; b += blockDim.x) {
    uint32_t v = lh[b];
    if (v) {
      atomicAdd(&gh[b], (unsigned long long)v);
      lh[b] = 0u;
    }
  }
}

// ---------------------------------------------------------------- k_sample
__device__ __forceinline__ uint32_t item_hash(uint64_t li) {
  uint64_t x = li * 0x9E3779B97F4A7C15ull;
  return (uint32_t)(x >> 33);
}

template <typename G>
__global__ __launch_bounds__(256) void k_sample(Workspace ws, const G* __restrict__ g,
                                                const float* __restrict__ e, int64_t ngroups) {
  __shared__ uint32_t lh[kSampleBins];
  for (int b = threadIdx.x; b < kSampleBins; b += blockDim.x) lh[b] = 0u;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int cur = -1;
  for (int64_t grp = blockIdx.x; grp < ngroups; grp += gridDim.x) {
    const int t = find_tensor_by_item(ws.td, ws.T, grp * kItemsPerGroup, cur < 0 ? 0 : cur);
    if (t != cur) {
      if (cur >= 0 && ws.td[cur].mode == kSampled) {
        __syncthreads();
        flush_lds_hist<kSampleBins>(lh, ws.shist + (int64_t)cur * kSampleBins);
        __syncthreads();
      }
      cur = t;
    }
    const TensorDesc d = ws.td[t];
    if (d.mode != kSampled) continue;
    const int64_t li = grp * kItemsPerGroup + wave - d.item_begin;
    if (li >= d.nitems) continue;
    const int64_t ioff = li * ws.item_len;
    const uint32_t len = (uint32_t)min((int64_t)ws.item_len, d.n - ioff);
    const uint32_t slen = min((uint32_t)d.sample_len, len);
    const uint32_t nphase = (len - slen) / kSampleGranule + 1u;
    const int64_t base = d.off + ioff + (int64_t)(item_hash((uint64_t)li) % nphase) * kSampleGranule;
    for (uint32_t j = lane; j < slen; j += 64) {
      const float acc = __fadd_rn(load_grad<G>(g, base + j), e[base + j]);
      atomicAdd(&lh[key_of(acc) >> kSampleShift], 1u);
    }
  }
  if (cur >= 0 && ws.td[cur].mode == kSampled) {
    __syncthreads();
    flush_lds_hist<kSampleBins>(lh, ws.shist + (int64_t)cur * kSampleBins);
  }
}

// ---------------------------------------------------------------- crossing search
// Largest bin b with sum_{j >= b} h[j] >= target; `above` = sum_{j > b} h[j].
// If the total is below target: b = 0. All threads of a 256-thread block call it;
// the result is valid in every thread.
template <int NB>
__device__ void find_from_top(const unsigned long long* __restrict__ h, unsigned long long target,
                              uint32_t& bin, unsigned long long& above) {
  constexpr int P = NB / 256;
  __shared__ unsigned long long part[256];
  __shared__ uint32_t s_bin;
  __shared__ unsigned long long s_above;
  unsigned long long mine = 0;
  for (int j = 0; j < P; ++j) mine += h[threadIdx.x * P + j];
  part[threadIdx.x] = mine;
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned long long acc = 0;
    int c = 255;
    for (; c > 0; --c) {
      if (acc + part[c] >= target) break;
      acc += part[c];
    }
    int b = c * P + P - 1;
    for (; b > c * P; --b) {
      if (acc + h[b] >= target) break;
      acc += h[b];
    }
    if (c == 0 && b == 0) { /* total may be below target: bin 0 either way */ }
    s_bin = (uint32_t)b;
    s_above = acc;
  }
  __syncthreads();
  bin = s_bin;
  above = s_above;
  __syncthreads();
}

__global__ __launch_bounds__(256) void k_sample_thresh(Workspace ws) {
  const int t = blockIdx.x;
  const TensorDesc d = ws.td[t];
  if (d.mode != kSampled) return;
  uint32_t bin;
  unsigned long long above;
  find_from_top<kSampleBins>(ws.shist + (int64_t)t * kSampleBins, (unsigned long long)d.sample_target,
                             bin, above);
  if (threadIdx.x == 0) ws.ts[t].t_lo = bin << kSampleShift;
}

// ---------------------------------------------------------------- k_main
// Append this lane's candidates of one row (4 consecutive elements per lane, lanes
// ascending) to the item's slots in ascending index order.
__device__ __forceinline__ void emit_row(bool c0, bool c1, bool c2, bool c3, f32x4 a, uint32_t rel,
                                         uint32_t& cnt, uint32_t cap, float* __restrict__ cv,
                                         uint32_t* __restrict__ cr) {
  const uint64_t m0 = __ballot(c0), m1 = __ballot(c1), m2 = __ballot(c2), m3 = __ballot(c3);
  if ((m0 | m1 | m2 | m3) == 0ull) return;
  uint32_t r = cnt + mbcnt64(m0) + mbcnt64(m1) + mbcnt64(m2) + mbcnt64(m3);
  if (c0) { if (r < cap) { cv[r] = a.x; cr[r] = rel; } ++r; }
  if (c1) { if (r < cap) { cv[r] = a.y; cr[r] = rel + 1u; } ++r; }
  if (c2) { if (r < cap) { cv[r] = a.z; cr[r] = rel + 2u; } ++r; }
  if (c3) { if (r < cap) { cv[r] = a.w; cr[r] = rel + 3u; } }
  cnt += (uint32_t)(__popcll(m0) + __popcll(m1) + __popcll(m2) + __popcll(m3));
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

template <typename G>
__global__ __launch_bounds__(256) void k_main(Workspace ws, const G* __restrict__ g, float* __restrict__ e) {
  __shared__ uint32_t lh[kSelBins];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t item = (int64_t)blockIdx.x * kItemsPerGroup + wave;
  const int t = find_tensor_by_item(ws.td, ws.T, (int64_t)blockIdx.x * kItemsPerGroup, 0);
  const TensorDesc d = ws.td[t];
  const bool dense = d.mode == kDense;  // uniform over the workgroup
  if (dense) {
    for (int b = threadIdx.x; b < kSelBins; b += 256) lh[b] = 0u;
    __syncthreads();
  }
  const int64_t li = item - d.item_begin;
  if (li < d.nitems) {
    const int64_t ioff = li * ws.item_len;
    const int64_t start = d.off + ioff;
    const uint32_t len = (uint32_t)min((int64_t)ws.item_len, d.n - ioff);
    const uint32_t t_lo = dense ? 0u : ws.ts[t].t_lo;
    const uint32_t cap = (uint32_t)ws.cap;
    float* __restrict__ cv = ws.cand_val + item * (int64_t)cap;
    uint32_t* __restrict__ cr = ws.cand_rel + item * (int64_t)cap;
    uint32_t cnt = 0;
    const G* gp = g + start;
    float* ep = e + start;
    uint32_t base = 0;
    const bool aligned = ((reinterpret_cast<uintptr_t>(gp) & GradVec<G>::kAlignMask) == 0) &&
                         ((reinterpret_cast<uintptr_t>(ep) & 15u) == 0);
    if (aligned) {
      for (; base + kWaveTile <= len; base += kWaveTile) {
        f32x4 gv[4], ev[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) gv[u] = GradVec<G>::load(gp + base + u * 256 + lane * 4);
#pragma unroll
        for (int u = 0; u < 4; ++u) ev[u] = *reinterpret_cast<const f32x4*>(ep + base + u * 256 + lane * 4);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          f32x4 a;
          a.x = __fadd_rn(gv[u].x, ev[u].x);
          a.y = __fadd_rn(gv[u].y, ev[u].y);
          a.z = __fadd_rn(gv[u].z, ev[u].z);
          a.w = __fadd_rn(gv[u].w, ev[u].w);
          __builtin_nontemporal_store(a, reinterpret_cast<f32x4*>(ep + base + u * 256 + lane * 4));
          const uint32_t k0 = key_of(a.x), k1 = key_of(a.y), k2 = key_of(a.z), k3 = key_of(a.w);
          if (dense) {
            atomicAdd(&lh[k0 >> 20], 1u);
            atomicAdd(&lh[k1 >> 20], 1u);
            atomicAdd(&lh[k2 >> 20], 1u);
            atomicAdd(&lh[k3 >> 20], 1u);
          } else {
            emit_row(k0 >= t_lo, k1 >= t_lo, k2 >= t_lo, k3 >= t_lo, a, base + u * 256 + lane * 4, cnt,
                     cap, cv, cr);
          }
        }
      }
    }
    // tail of the item, or the whole item when its addresses are not 16-byte aligned
    for (uint32_t j0 = base; j0 < len; j0 += 64) {
      const uint32_t j = j0 + lane;
      const bool valid = j < len;
      float a = 0.0f;
      if (valid) {
        a = __fadd_rn(load_grad<G>(gp, j), ep[j]);
        ep[j] = a;
      }
      const uint32_t key = key_of(a);
      if (dense) {
        if (valid) atomicAdd(&lh[key >> 20], 1u);
      } else {
        const bool c = valid && key >= t_lo;
        const uint64_t m = __ballot(c);
        if (m) {
          const uint32_t r = cnt + mbcnt64(m);
          if (c && r < cap) { cv[r] = a; cr[r] = j; }
          cnt += (uint32_t)__popcll(m);
        }
      }
    }
    if (!dense && lane == 0) {
      ws.item_cnt[item] = min(cnt, cap);
      if (cnt > cap) ws.ts[t].overflow = 1u;
      if (cnt) atomicAdd(&ws.ts[t].cand_total, (unsigned long long)cnt);
    }
  } else if (!dense && lane == 0) {
    ws.item_cnt[item] = 0u;
  }
  if (dense) {
    __syncthreads();
    flush_lds_hist<kSelBins>(lh, ws.hist + (int64_t)t * kSelBins);
  }
}

// ---------------------------------------------------------------- source of the select passes
// After k_main an item is read either from its candidate slots (sampled tensor, fast path
// holds) or from the dense residual, which now holds acc.
struct ItemSrc {
  const float* val;     // values, ascending index order
  const uint32_t* rel;  // offsets inside the item (null: offset = position)
  uint32_t len;
};

__device__ __forceinline__ ItemSrc item_source(const Workspace& ws, const TensorDesc& d, bool use_cand,
                                               int64_t item, const float* e) {
  ItemSrc s;
  const int64_t li = item - d.item_begin;
  if (li >= d.nitems) { s.val = nullptr; s.rel = nullptr; s.len = 0; return s; }
  if (use_cand) {
    s.val = ws.cand_val + item * (int64_t)ws.cap;
    s.rel = ws.cand_rel + item * (int64_t)ws.cap;
    s.len = ws.item_cnt[item];
  } else {
    const int64_t ioff = li * ws.item_len;
    s.val = e + d.off + ioff;
    s.rel = nullptr;
    s.len = (uint32_t)min((int64_t)ws.item_len, d.n - ioff);
  }
  return s;
}

// ---------------------------------------------------------------- k_hist
__global__ __launch_bounds__(256) void k_hist(Workspace ws, int level, const float* __restrict__ e,
                                              int64_t ngroups) {
  __shared__ uint32_t lh[kSelBins];
  for (int b = threadIdx.x; b < kSelBins; b += 256) lh[b] = 0u;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int shift = sel_shift(level);
  const uint32_t mask = (1u << sel_bits(level)) - 1u;
  const int pshift = shift + sel_bits(level);  // bits above this digit must match the prefix
  int cur = -1;
  for (int64_t grp = blockIdx.x; grp < ngroups; grp += gridDim.x) {
    const int t = find_tensor_by_item(ws.td, ws.T, grp * kItemsPerGroup, cur < 0 ? 0 : cur);
    if (t != cur) {
      if (cur >= 0) {
        __syncthreads();
        flush_lds_hist<kSelBins>(lh, ws.hist + (int64_t)cur * kSelBins);
        __syncthreads();
      }
      cur = t;
    }
    const TensorDesc d = ws.td[t];
    const TensorState st = ws.ts[t];
    const bool use_cand = d.mode == kSampled && !fast_path_failed(st, d);
    if (level == 0 && d.mode == kDense) continue;  // k_main already built this digit
    const ItemSrc s = item_source(ws, d, use_cand, grp * kItemsPerGroup + wave, e);
    const uint32_t want = (level == 0) ? 0u : (st.prefix >> pshift);
    for (uint32_t j = lane; j < s.len; j += 64) {
      const uint32_t key = key_of(s.val[j]);
      if (level == 0 || (key >> pshift) == want) atomicAdd(&lh[(key >> shift) & mask], 1u);
    }
  }
  if (cur >= 0) {
    __syncthreads();
    flush_lds_hist<kSelBins>(lh, ws.hist + (int64_t)cur * kSelBins);
  }
}

// ---------------------------------------------------------------- k_select_scan
__global__ __launch_bounds__(256) void k_select_scan(Workspace ws, int level) {
  const int t = blockIdx.x;
  const TensorDesc d = ws.td[t];
  unsigned long long* h = ws.hist + (int64_t)t * kSelBins;
  const unsigned long long k_rem = (level == 0) ? (unsigned long long)d.k : ws.ts[t].k_rem;
  uint32_t bin;
  unsigned long long above;
  find_from_top<kSelBins>(h, k_rem, bin, above);
  for (int b = threadIdx.x; b < kSelBins; b += 256) h[b] = 0ull;  // ready for the next digit
  if (threadIdx.x == 0) {
    ws.ts[t].k_rem = k_rem - above;
    const uint32_t p = (level == 0) ? 0u : ws.ts[t].prefix;
    ws.ts[t].prefix = p | (bin << sel_shift(level));
  }
}

// ---------------------------------------------------------------- k_count
__global__ __launch_bounds__(256) void k_count(Workspace ws, const float* __restrict__ e) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t item = (int64_t)blockIdx.x * kItemsPerGroup + wave;
  const int t = find_tensor_by_item(ws.td, ws.T, (int64_t)blockIdx.x * kItemsPerGroup, 0);
  const TensorDesc d = ws.td[t];
  const TensorState st = ws.ts[t];
  const bool use_cand = d.mode == kSampled && !fast_path_failed(st, d);
  const ItemSrc s = item_source(ws, d, use_cand, item, e);
  const uint32_t thr = st.prefix;
  uint32_t gt = 0, eq = 0;
  for (uint32_t j0 = 0; j0 < s.len; j0 += 64) {
    const uint32_t j = j0 + lane;
    const bool valid = j < s.len;
    const uint32_t key = valid ? key_of(s.val[j]) : 0u;
    gt += (uint32_t)__popcll(__ballot(valid && key > thr));
    eq += (uint32_t)__popcll(__ballot(valid && key == thr));
  }
  if (lane == 0) {
    ws.item_gt[item] = gt;
    ws.item_eq[item] = eq;
  }
}

// ---------------------------------------------------------------- k_item_scan
// Exclusive prefix sums of item_gt / item_eq over the item slots of one tensor.
constexpr int kScanThreads = 1024;
constexpr int kScanPer = 8;
__global__ __launch_bounds__(kScanThreads) void k_item_scan(Workspace ws) {
  __shared__ long long wsum_g[kScanThreads / 64], wsum_e[kScanThreads / 64];
  __shared__ long long carry_g, carry_e;
  const int t = blockIdx.x;
  const TensorDesc d = ws.td[t];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (threadIdx.x == 0) { carry_g = 0; carry_e = 0; }
  __syncthreads();
  const int64_t nslots = d.item_end - d.item_begin;
  for (int64_t c0 = 0; c0 < nslots; c0 += (int64_t)kScanThreads * kScanPer) {
    const int64_t first = d.item_begin + c0 + (int64_t)threadIdx.x * kScanPer;
    uint32_t vg[kScanPer], ve[kScanPer];
    long long sg = 0, se = 0;
#pragma unroll
    for (int j = 0; j < kScanPer; ++j) {
      const bool in = first + j < d.item_end;
      vg[j] = in ? ws.item_gt[first + j] : 0u;
      ve[j] = in ? ws.item_eq[first + j] : 0u;
      sg += vg[j];
      se += ve[j];
    }
    // inclusive scan across the wavefront
    long long ig = sg, ie = se;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const long long ug = __shfl_up(ig, off), ue = __shfl_up(ie, off);
      if (lane >= off) { ig += ug; ie += ue; }
    }
    if (lane == 63) { wsum_g[wave] = ig; wsum_e[wave] = ie; }
    __syncthreads();
    long long bg = carry_g, be = carry_e;
    for (int w = 0; w < wave; ++w) { bg += wsum_g[w]; be += wsum_e[w]; }
    long long xg = bg + ig - sg, xe = be + ie - se;  // exclusive prefix of this thread's first slot
#pragma unroll
    for (int j = 0; j < kScanPer; ++j) {
      if (first + j < d.item_end) {
        ws.item_goff[first + j] = xg;
        ws.item_eoff[first + j] = xe;
      }
      xg += vg[j];
      xe += ve[j];
    }
    __syncthreads();
    if (threadIdx.x == kScanThreads - 1) { carry_g = xg; carry_e = xe; }
    __syncthreads();
  }
}

// ---------------------------------------------------------------- k_emit
template <typename I>
__global__ __launch_bounds__(256) void k_emit(Workspace ws, const float* __restrict__ e,
                                              I* __restrict__ out_idx) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t item = (int64_t)blockIdx.x * kItemsPerGroup + wave;
  const int t = find_tensor_by_item(ws.td, ws.T, (int64_t)blockIdx.x * kItemsPerGroup, 0);
  const TensorDesc d = ws.td[t];
  const TensorState st = ws.ts[t];
  const bool use_cand = d.mode == kSampled && !fast_path_failed(st, d);
  const ItemSrc s = item_source(ws, d, use_cand, item, e);
  if (s.len == 0) return;
  const uint32_t thr = st.prefix;
  const long long quota = (long long)st.k_rem;
  long long G = ws.item_goff[item], E = ws.item_eoff[item];
  const int64_t item_first = d.off + (item - d.item_begin) * ws.item_len;  // flat index of offset 0
  for (uint32_t j0 = 0; j0 < s.len; j0 += 64) {
    const uint32_t j = j0 + lane;
    const bool valid = j < s.len;
    const float v = valid ? s.val[j] : 0.0f;
    const uint32_t key = key_of(v);
    const bool isgt = valid && key > thr, iseq = valid && key == thr;
    const uint64_t mg = __ballot(isgt), me = __ballot(iseq);
    const long long grank = G + mbcnt64(mg), erank = E + mbcnt64(me);
    const bool keep = isgt || (iseq && erank < quota);
    if (keep) {
      const long long pos = d.kprefix + grank + (erank < quota ? erank : quota);
      const uint32_t rel = s.rel ? s.rel[j] : j;
      out_idx[pos] = (I)(item_first + rel);
      ws.kept_val[pos] = v;
    }
    G += __popcll(mg);
    E += __popcll(me);
  }
}

// ---------------------------------------------------------------- k_quant
// One workgroup per block of `block` consecutive kept entries of one tensor.
template <typename I>
__global__ __launch_bounds__(256) void k_quant(Workspace ws, float* __restrict__ e,
                                               const I* __restrict__ idx, int8_t* __restrict__ q,
                                               float* __restrict__ scales, int32_t block) {
  __shared__ uint32_t s_amax;
  const int64_t gb = blockIdx.x;
  int t = 0;
  if (ws.T > 1) {  // largest t with sprefix <= gb
    int lo = 0, hi = ws.T - 1;
    while (lo < hi) {
      int mid = (lo + hi + 1) >> 1;
      if (ws.td[mid].sprefix <= gb) lo = mid; else hi = mid - 1;
    }
    t = lo;
  }
  const TensorDesc d = ws.td[t];
  const int64_t j0 = d.kprefix + (gb - d.sprefix) * block;
  const int64_t j1 = min(d.kprefix + d.k, j0 + block);
  if (threadIdx.x == 0) s_amax = 0u;
  __syncthreads();
  uint32_t m = 0;
  for (int64_t j = j0 + threadIdx.x; j < j1; j += blockDim.x) m = max(m, key_of(ws.kept_val[j]));
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off));
  if ((threadIdx.x & 63) == 0) atomicMax(&s_amax, m);
  __syncthreads();
  const uint32_t akey = s_amax;
  const bool finite = akey < 0x7F800000u;
  float s = __fdiv_rn(__uint_as_float(akey), 127.0f);
  if (!finite || !(s >= 1.17549435e-38f)) s = 0.0f;
  if (threadIdx.x == 0) {
    scales[gb] = s;
    if (!finite) ws.flags[0] = 1u;
  }
  for (int64_t j = j0 + threadIdx.x; j < j1; j += blockDim.x) {
    const float v = ws.kept_val[j];
    int code = 0;
    if (s != 0.0f) {
      float r = rintf(__fdiv_rn(v, s));
      r = fminf(fmaxf(r, -127.0f), 127.0f);
      code = (int)r;
    }
    q[j] = (int8_t)code;
    if (finite) {
      const float dq = __fmul_rn((float)code, s);
      e[(int64_t)idx[j]] = __fsub_rn(v, dq);
    }
  }
}

inline int clamp_grid(int64_t want, int64_t cap) { return (int)(want < 1 ? 1 : (want > cap ? cap : want)); }
inline int64_t ngroups_of(const Workspace& ws) { return ws.nitem_slots / kItemsPerGroup; }

}  // namespace

void launch_init(const Workspace& ws, hipStream_t s) {
  const int64_t work = (int64_t)ws.T * kSampleBins;
  hipLaunchKernelGGL(k_init, dim3(clamp_grid((work + 255) / 256, 2048)), dim3(256), 0, s, ws);
}

void launch_sample(const Workspace& ws, const void* g, int dtype, const float* e, hipStream_t s) {
  const int64_t ng = ngroups_of(ws);
  const dim3 grid(clamp_grid(ng, 2048));
  if (dtype == 0)
    hipLaunchKernelGGL(k_sample<float>, grid, dim3(256), 0, s, ws, (const float*)g, e, ng);
  else
    hipLaunchKernelGGL(k_sample<uint16_t>, grid, dim3(256), 0, s, ws, (const uint16_t*)g, e, ng);
}

void launch_sample_thresh(const Workspace& ws, hipStream_t s) {
  hipLaunchKernelGGL(k_sample_thresh, dim3(ws.T), dim3(256), 0, s, ws);
}

void launch_main(const Workspace& ws, const void* g, int dtype, float* e, hipStream_t s) {
  const dim3 grid((unsigned)ngroups_of(ws));
  if (dtype == 0)
    hipLaunchKernelGGL(k_main<float>, grid, dim3(256), 0, s, ws, (const float*)g, e);
  else
    hipLaunchKernelGGL(k_main<uint16_t>, grid, dim3(256), 0, s, ws, (const uint16_t*)g, e);
}

void launch_hist(const Workspace& ws, int level, const float* e, hipStream_t s) {
  const int64_t ng = ngroups_of(ws);
  hipLaunchKernelGGL(k_hist, dim3(clamp_grid(ng, 2048)), dim3(256), 0, s, ws, level, e, ng);
}

void launch_select_scan(const Workspace& ws, int level, hipStream_t s) {
  hipLaunchKernelGGL(k_select_scan, dim3(ws.T), dim3(256), 0, s, ws, level);
}

void launch_count(const Workspace& ws, const float* e, hipStream_t s) {
  hipLaunchKernelGGL(k_count, dim3((unsigned)ngroups_of(ws)), dim3(256), 0, s, ws, e);
}

void launch_item_scan(const Workspace& ws, hipStream_t s) {
  hipLaunchKernelGGL(k_item_scan, dim3(ws.T), dim3(kScanThreads), 0, s, ws);
}

void launch_emit(const Workspace& ws, const float* e, const OutBuf& out, hipStream_t s) {
  const dim3 grid((unsigned)ngroups_of(ws));
  if (out.index_bits == 32)
    hipLaunchKernelGGL(k_emit<uint32_t>, grid, dim3(256), 0, s, ws, e, (uint32_t*)out.indices);
  else
    hipLaunchKernelGGL(k_emit<unsigned long long>, grid, dim3(256), 0, s, ws, e,
                       (unsigned long long*)out.indices);
}

void launch_quant(const Workspace& ws, float* e, const OutBuf& out, int64_t total_blocks, hipStream_t s) {
  int threads = out.block >= 256 ? 256 : ((out.block + 63) / 64) * 64;
  const dim3 grid((unsigned)total_blocks);
  if (out.index_bits == 32)
    hipLaunchKernelGGL(k_quant<uint32_t>, grid, dim3(threads), 0, s, ws, e, (const uint32_t*)out.indices,
                       out.q, out.scales, out.block);
  else
    hipLaunchKernelGGL(k_quant<unsigned long long>, grid, dim3(threads), 0, s, ws, e,
                       (const unsigned long long*)out.indices, out.q, out.scales, out.block);
}

}  // namespace gc
