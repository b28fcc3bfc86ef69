// Compress side: error-feedback accumulate, exact magnitude top-k, per-block int8
// codes and the fused residual write-back (paper Sec. III.B, Eq. 11), for gfx950.
//
// Shape of the computation (one call = one worker's step over T tensors)
//   1. k_sample / k_sample_thresh   read one 256-element granule out of every `stride`,
//        form acc = g + e there, histogram the top 13 key bits in LDS and pick a candidate
//        threshold t_lo that, with overwhelming probability, lies below the k-th largest key.
//   2. k_main   THE streaming pass, the only one that touches every element: a workgroup
//        streams one group of 1024 consecutive elements with 128-bit loads, writes
//        acc = g + e over e, and appends every entry with key >= t_lo, in ascending index
//        order (wavefront ballots + a 4-entry LDS prefix), to the group's candidate slots.
//        Workgroups are short-lived and few per CU: HBM sees a narrow window of addresses
//        that moves through the arrays once, which is what gets closest to its streaming rate.
//   3. k_group_scan / k_route / k_gather   prefix-sum the groups' counts and pack all
//        candidates of a tensor into one dense ascending array.
//   4. k_hist / k_select_scan (x3)   exact radix select (LDS histograms per workgroup) of the
//        k-th largest key T and the tie quota, over the dense candidates.
//   5. k_count / k_chunk_scan / k_emit   ordered compaction (wavefront ballot + prefix) of the
//        kept entries: key > T, or key == T among the first `quota` such entries.
//   6. k_quant   per block of kept entries: amax, scale, int8 codes, and the residual at the
//        kept positions, acc - q*s (Eq. 11 with ghat = q*s).
//   On the dense route of a single tensor, a counting pass around a guessed tie key (tie_spec_count,
//   inside k_gather's launch) replaces steps 4 and k_count when the guess verifies exactly.
//   Small or dense tensors skip 1 and 3: steps 4-5 then read the residual itself (it holds
//   acc after step 2). A sampled tensor whose candidates turn out too few or too many takes
//   that same dense route, decided on the device; candidates clustered beyond a group's slots
//   are re-read from the residual by the gather. The result never depends on the sample, only
//   the time does.
#include <algorithm>

#include "gc_internal.h"

namespace gc {
namespace {

// Largest t in [0, T) with begin(t) <= x (begin is non-decreasing, begin(0) <= x).
template <typename F>
__device__ __forceinline__ int find_last_le(int T, long long x, int hint, F begin) {
  if (T == 1) return 0;
  if (begin(hint) <= x && (hint + 1 == T || begin(hint + 1) > x)) return hint;
  int lo = 0, hi = T - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (begin(mid) <= x) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// The same inside a known range of tensors [t_lo, t_hi] (begin(t_lo) <= x, and x lies before the
// tensor after t_hi): the search of a position whose neighbourhood has been located already.
template <typename F>
__device__ __forceinline__ int find_last_le_in(int t_lo, int t_hi, long long x, F begin) {
  int lo = t_lo, hi = t_hi;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (begin(mid) <= x) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// Sum over the block of one value per thread (blockDim.x a multiple of 64, <= 1024).
__device__ __forceinline__ unsigned long long block_sum(unsigned long long v, unsigned long long* sh) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[wave] = v;
  __syncthreads();
  unsigned long long t = 0;
  for (int w = 0; w < nw; ++w) t += sh[w];
  return t;
}

// ---------------------------------------------------------------- LDS histogram flush
template <int NB>
__device__ __forceinline__ void flush_lds_hist(uint32_t* lh, unsigned long long* gh) {
  for (int b = threadIdx.x; b < NB; b += blockDim.x) {
    const uint32_t v = lh[b];
    if (v) {
      atomicAdd(&gh[b], (unsigned long long)v);
      lh[b] = 0u;
    }
  }
}

// One count per lane into an LDS histogram. When every participating lane of the wavefront hits the
// same bin (long runs of equal keys: ties, exact zeros) a single lane adds the whole count: 64
// atomics on one LDS address would be executed one after the other.
__device__ __forceinline__ void hist_add(uint32_t* lh, bool on, uint32_t bin) {
  const uint64_t act = __ballot(on);
  if (act == 0ull) return;
  const int first = __ffsll((unsigned long long)act) - 1;
  const uint32_t b0 = (uint32_t)__builtin_amdgcn_readlane((int)bin, first);
  if (__ballot(on && bin != b0) == 0ull) {
    if ((int)(threadIdx.x & 63) == first) atomicAdd(&lh[b0], (uint32_t)__popcll(act));
  } else if (on) {
    atomicAdd(&lh[bin], 1u);
  }
}

// ---------------------------------------------------------------- k_sample
__device__ __forceinline__ uint32_t mix_hash(uint64_t x) {
  x *= 0x9E3779B97F4A7C15ull;
  return (uint32_t)(x >> 33);
}

// One sampled granule as a wavefront sees it: where it lies, and its 256 values once loaded.
template <typename G>
struct SampleItem {
  int t;          // tensor (uniform over the workgroup), -1: no slot
  bool active;    // this wavefront has a granule in the slot quadruple
  float gv[4], ev[4];  // the lane's 4 gradient and residual values, as loaded (added when consumed)
};

template <typename G>
__device__ __forceinline__ SampleItem<G> sample_fetch(const Workspace& ws, const G* __restrict__ g,
                                                      const float* __restrict__ e, int64_t s0, int64_t s_end,
                                                      int hint, int lane, int wave) {
  SampleItem<G> it;
  it.t = -1;
  it.active = false;
#pragma unroll
  for (int c = 0; c < 4; ++c) it.gv[c] = it.ev[c] = 0.0f;
  if (s0 >= s_end) return it;
  it.t = find_last_le(ws.T, s0, hint < 0 ? 0 : hint, [&](int i) { return (long long)ws.desc(i).sgran_begin; });
  const TensorDesc d = ws.desc(it.t);
  const int64_t ls = s0 + wave - d.sgran_begin;  // sgran_begin is a multiple of 4 and nsgran padded
  if (ls >= d.nsgran) return it;
  it.active = true;
  const int64_t gran = ls * d.sample_stride + (int64_t)(mix_hash((uint64_t)ls) % (uint32_t)d.sample_stride);
  const int64_t base = d.off + gran * kSampleGranule;
  const G* gp = g + base;
  const float* ep = e + base;
  const bool aligned = ((reinterpret_cast<uintptr_t>(gp) & GradVec<G>::kAlignMask) == 0) &&
                       ((reinterpret_cast<uintptr_t>(ep) & 15u) == 0);
  if (aligned) {
    const f32x4 gv = GradVec<G>::load(gp + lane * 4);
    const f32x4 ev = *reinterpret_cast<const f32x4*>(ep + lane * 4);
    it.gv[0] = gv.x; it.gv[1] = gv.y; it.gv[2] = gv.z; it.gv[3] = gv.w;
    it.ev[0] = ev.x; it.ev[1] = ev.y; it.ev[2] = ev.z; it.ev[3] = ev.w;
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int j = c * 64 + lane;
      it.gv[c] = load_grad<G>(gp, j);
      it.ev[c] = ep[j];
    }
  }
  return it;
}

template <typename G>
__global__ __launch_bounds__(256) void k_sample(Workspace ws, const G* __restrict__ g,
                                                const float* __restrict__ e) {
  __shared__ uint32_t lh[kSampleBins];
  for (int b = threadIdx.x; b < kSampleBins; b += 256) lh[b] = 0u;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int cur = -1;
  // A workgroup takes 4 consecutive sampled-granule slots per step, one per wavefront. Every
  // tensor's slots start at a multiple of 4 and are padded to a multiple of 4, so one step never
  // mixes tensors and the LDS histogram can be flushed when the tensor changes. Each workgroup
  // takes one contiguous run of slots, so it meets few tensors. Two steps are fetched before the
  // first is histogrammed: the run is a chain of dependent round trips to memory otherwise.
  const int64_t per = ((ws.nsgran / 4 + gridDim.x - 1) / gridDim.x) * 4;
  const int64_t s_end = min(ws.nsgran, ((int64_t)blockIdx.x + 1) * per);
  auto consume = [&](const SampleItem<G>& it) {
    if (it.t < 0) return;  // uniform over the workgroup
    if (it.t != cur) {
      if (cur >= 0) {
        __syncthreads();
        flush_lds_hist<kSampleBins>(lh, ws.shist + (int64_t)cur * kSampleBins);
        __syncthreads();
      }
      cur = it.t;
    }
    if (it.active) {
#pragma unroll
      for (int c = 0; c < 4; ++c) atomicAdd(&lh[key_of(__fadd_rn(it.gv[c], it.ev[c])) >> kSampleShift], 1u);
    }
  };
  for (int64_t s0 = (int64_t)blockIdx.x * per; s0 < s_end; s0 += 8) {
    const SampleItem<G> a = sample_fetch<G>(ws, g, e, s0, s_end, cur, lane, wave);
    const SampleItem<G> b = sample_fetch<G>(ws, g, e, s0 + 4, s_end, a.t, lane, wave);
    consume(a);
    consume(b);
  }
  if (cur >= 0) {
    __syncthreads();
    flush_lds_hist<kSampleBins>(lh, ws.shist + (int64_t)cur * kSampleBins);
  }
}

// ---------------------------------------------------------------- crossing search
// Largest bin b with sum_{j >= b} h[j] >= target; `above` = sum_{j > b} h[j].
// If the total is below target: b = 0. All threads of the block call it (blockDim.x = NT);
// the result is valid in every thread. h may live in global memory or in LDS.
template <int NB, int NT, typename H>
__device__ void find_from_top(const H* __restrict__ h, unsigned long long target, uint32_t& bin,
                              unsigned long long& above) {
  constexpr int P = NB / NT;  // bins per thread
  constexpr int NW = NT / 64;
  __shared__ unsigned long long s_wsum[NW];
  __shared__ int s_wcnt[NW];
  __shared__ uint32_t s_bin;
  __shared__ unsigned long long s_above;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  unsigned long long mine = 0;
#pragma unroll
  for (int j = 0; j < P; ++j) mine += (unsigned long long)h[threadIdx.x * P + j];
  // from_here = sum over this thread's bins and all bins above them: a suffix sum over the threads
  unsigned long long incl = mine;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned long long u = __shfl_down(incl, off);
    if (lane + off < 64) incl += u;
  }
  if (lane == 0) s_wsum[wave] = incl;
  __syncthreads();
  unsigned long long after = 0;
  for (int w = wave + 1; w < NW; ++w) after += s_wsum[w];
  const unsigned long long from_here = incl + after;
  // from_here falls with the thread number, so the threads that still reach the target are
  // 0 .. c, c being the thread whose bins hold the crossing
  const uint64_t reach = __ballot(from_here >= target);
  if (lane == 0) s_wcnt[wave] = __popcll(reach);
  __syncthreads();
  int c = -1;
  for (int w = 0; w < NW; ++w) c += s_wcnt[w];
  if (c < 0) c = 0;
  if ((int)threadIdx.x == c) {
    unsigned long long acc = from_here - mine;  // everything above this thread's bins
    int b = c * P + P - 1;
    for (; b > c * P; --b) {
      const unsigned long long hb = (unsigned long long)h[b];
      if (acc + hb >= target) break;
      acc += hb;
    }
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
  const TensorDesc d = ws.desc(t);
  if (d.mode != kSampled) return;
  uint32_t bin;
  unsigned long long above;
  unsigned long long* sh = ws.shist + (int64_t)t * kSampleBins;
  find_from_top<kSampleBins, 256>(sh, (unsigned long long)d.sample_target, bin, above);
  if (threadIdx.x == 0) ws.ts[t].t_lo = bin << kSampleShift;
  for (int b = threadIdx.x; b < kSampleBins; b += 256) sh[b] = 0ull;  // left zeroed for the next call
}

// ---------------------------------------------------------------- k_main
// The prologue is kept short on purpose: a workgroup lives for one group only, so every
// dependent load in front of its first streaming load shows up in the achieved bandwidth. A
// single tensor needs kernel arguments only; several tensors cost one 16-byte record per group.
template <typename G>
__global__ __launch_bounds__(256) void k_main(Workspace ws, const G* __restrict__ g, float* __restrict__ e,
                                              const GroupRec* __restrict__ recs, long long n_single,
                                              int sampled_single) {
  // dynamic LDS: staging for the group's candidates; its size also bounds how many workgroups
  // share a CU (the launcher asks for more than the staging needs on purpose)
  extern __shared__ __align__(16) char lds_dyn[];
  __shared__ uint32_t wcnt[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // Consecutive workgroups are dispatched to different compute dies (8 of them, round robin).
  // Each die is given runs of kXcdRun consecutive groups, so the lines (and pages) one die's L2
  // and TLB see are contiguous, while all dies together still move one window through memory.
  const int64_t grp = xcd_run_index(blockIdx.x);
  if (grp >= ws.ngroups) return;  // the grid is padded to whole rounds of runs
  long long gstart;  // first element of the group in the flat arrays
  int glen, t;
  bool sampled;
  if (recs == nullptr) {
    gstart = grp * (long long)kGroup;
    glen = (int)min((long long)kGroup, n_single - gstart);
    t = 0;
    sampled = sampled_single != 0;
  } else {
    const GroupRec r = recs[grp];
    gstart = r.start;
    glen = r.len;
    t = (int)(r.tensor & 0x7FFFFFFFu);
    sampled = (r.tensor >> 31) != 0u;
  }
  const int wstart = wave * kWaveTile;
  const int wlen = max(0, min(kWaveTile, glen - wstart));
  // The candidate threshold is fetched with a vector load issued AFTER the streaming loads, so
  // that its latency hides behind theirs instead of delaying them (a scalar load would be
  // waited for first). The zero offset is opaque to the compiler on purpose.
  uint32_t lane_zero;
  asm volatile("v_mov_b32 %0, 0" : "=v"(lane_zero));
  const uint32_t* t_lo_ptr = &ws.ts[t].t_lo + lane_zero;
  uint32_t t_lo = 0xFFFFFFFFu;  // no key reaches 0xFFFFFFFF: a dense tensor gathers no candidates
  const G* gp = g + gstart + wstart;
  float* ep = e + gstart + wstart;
  const bool vec = wlen == kWaveTile && ((reinterpret_cast<uintptr_t>(gp) & GradVec<G>::kAlignMask) == 0) &&
                   ((reinterpret_cast<uintptr_t>(ep) & 15u) == 0);
  f32x4 a[kRows];
  uint32_t rank[kRows];
  uint32_t flags = 0u, mycnt = 0u;
  if (vec) {
    f32x4 gv[kRows], ev[kRows];
#pragma unroll
    for (int u = 0; u < kRows; ++u) gv[u] = GradVec<G>::load(gp + u * 256 + lane * 4);
#pragma unroll
    for (int u = 0; u < kRows; ++u)  // read once, then overwritten: non-temporal like g (measured +4 %)
      ev[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(ep + u * 256 + lane * 4));
    if (sampled) t_lo = *t_lo_ptr;
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
      a[u].x = __fadd_rn(gv[u].x, ev[u].x);
      a[u].y = __fadd_rn(gv[u].y, ev[u].y);
      a[u].z = __fadd_rn(gv[u].z, ev[u].z);
      a[u].w = __fadd_rn(gv[u].w, ev[u].w);
      __builtin_nontemporal_store(a[u], reinterpret_cast<f32x4*>(ep + u * 256 + lane * 4));
      const bool c0 = key_of(a[u].x) >= t_lo, c1 = key_of(a[u].y) >= t_lo, c2 = key_of(a[u].z) >= t_lo,
                 c3 = key_of(a[u].w) >= t_lo;
      const uint64_t m0 = __ballot(c0), m1 = __ballot(c1), m2 = __ballot(c2), m3 = __ballot(c3);
      rank[u] = mycnt + mbcnt64(m0) + mbcnt64(m1) + mbcnt64(m2) + mbcnt64(m3);
      flags |= ((uint32_t)c0 | ((uint32_t)c1 << 1) | ((uint32_t)c2 << 2) | ((uint32_t)c3 << 3)) << (4 * u);
      mycnt += (uint32_t)(__popcll(m0) + __popcll(m1) + __popcll(m2) + __popcll(m3));
    }
  } else {
    // tail group of a tensor, or addresses that are not 16-byte aligned: one element per lane
    if (sampled) t_lo = *t_lo_ptr;
    for (int j0 = 0; j0 < wlen; j0 += 64) {
      const int j = j0 + lane;
      bool c = false;
      if (j < wlen) {
        const float acc = __fadd_rn(load_grad<G>(gp, j), ep[j]);
        ep[j] = acc;
        c = key_of(acc) >= t_lo;
      }
      mycnt += (uint32_t)__popcll(__ballot(c));
    }
  }
  if (!sampled) return;  // uniform over the workgroup: a dense tensor gathers no candidates
  if (lane == 0) wcnt[wave] = mycnt;
  __syncthreads();
  uint32_t before = 0u, tot = 0u;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const uint32_t c = wcnt[w];
    if (w < wave) before += c;
    tot += c;
  }
  // Candidates are staged in LDS in ascending index order and leave the workgroup as whole
  // 128-byte lines of records, padded with zero records: scattered 8-byte stores would become
  // partial-line writes in HBM and cost more than the bytes they carry.
  const uint32_t cap = (uint32_t)ws.cap;
  uint2* stage = reinterpret_cast<uint2*>(lds_dyn);
  if (tot) {
    if (vec) {
      if (flags) {
#pragma unroll
        for (int u = 0; u < kRows; ++u) {
          const uint32_t f = (flags >> (4 * u)) & 15u;
          if (f) {
            uint32_t r = before + rank[u];
            const uint32_t rel = (uint32_t)(wstart + u * 256 + lane * 4);
            if (f & 1u) { if (r < cap) stage[r] = make_uint2(__float_as_uint(a[u].x), rel); ++r; }
            if (f & 2u) { if (r < cap) stage[r] = make_uint2(__float_as_uint(a[u].y), rel + 1u); ++r; }
            if (f & 4u) { if (r < cap) stage[r] = make_uint2(__float_as_uint(a[u].z), rel + 2u); ++r; }
            if (f & 8u) { if (r < cap) stage[r] = make_uint2(__float_as_uint(a[u].w), rel + 3u); }
          }
        }
      }
    } else if (mycnt) {
      // second look at what this wave just wrote (acc is in e now)
      uint32_t r0 = before;
      for (int j0 = 0; j0 < wlen; j0 += 64) {
        const int j = j0 + lane;
        float acc = 0.0f;
        bool c = false;
        if (j < wlen) {
          acc = ep[j];
          c = key_of(acc) >= t_lo;
        }
        const uint64_t m = __ballot(c);
        const uint32_t r = r0 + mbcnt64(m);
        if (c && r < cap) stage[r] = make_uint2(__float_as_uint(acc), (uint32_t)(wstart + j));
        r0 += (uint32_t)__popcll(m);
      }
    }
    __syncthreads();  // tot is uniform over the workgroup
  }
  // The group's count goes to a compact array (plain 4-byte stores of neighbouring workgroups
  // combine in L2); a group without candidates writes no records at all.
  if (threadIdx.x == 0) ws.grp_cnt[grp] = tot;
  const uint32_t kept = min(tot, cap);
  // whole lines; with at most 8 slots per group two neighbouring groups share a 128-byte line and
  // each writes its half (they run on the same die at about the same time, so the halves meet in L2)
  const uint32_t line = (uint32_t)(ws.slot_stride < kSlotLine ? ws.slot_stride : kSlotLine);
  const uint32_t nout = (kept + line - 1) & ~(line - 1);
  uint2* __restrict__ dst = ws.slots + grp * (int64_t)ws.slot_stride;
  for (uint32_t j = threadIdx.x; j < nout; j += 256) dst[j] = j < kept ? stage[j] : make_uint2(0u, 0u);
}

// ---------------------------------------------------------------- block-wise exclusive scan
// Exclusive prefix of v[0..n) inside block `b` of kScanBlock entries, on top of the sum of all
// earlier blocks (taken from the block sums `part`). 256 threads, 4 entries each; the scanned
// values of the block are also left in `lds_out` (kScanBlock + 1 entries, last = block end).
__device__ __forceinline__ void scan_block(const uint32_t* __restrict__ v, int64_t n,
                                           const unsigned long long* __restrict__ part, int64_t b,
                                           long long* __restrict__ out, long long* lds_out,
                                           unsigned long long* sh) {
  unsigned long long mine = 0;
  for (int64_t i = threadIdx.x; i < b; i += blockDim.x) mine += part[i];
  const long long base = (long long)block_sum(mine, sh);
  const int64_t i0 = b * kScanBlock + (int64_t)threadIdx.x * 4;
  uint32_t c[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) c[j] = (i0 + j < n) ? v[i0 + j] : 0u;
  const long long s = (long long)c[0] + c[1] + c[2] + c[3];
  long long incl = s;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const long long u = __shfl_up(incl, off);
    if (lane >= off) incl += u;
  }
  __syncthreads();
  if (lane == 63) sh[wave] = (unsigned long long)incl;
  __syncthreads();
  long long x = base + incl - s;
  for (int w = 0; w < wave; ++w) x += (long long)sh[w];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (i0 + j < n) out[i0 + j] = x;
    lds_out[threadIdx.x * 4 + j] = x;
    x += c[j];
  }
  if (threadIdx.x == 255) lds_out[kScanBlock] = x;
  __syncthreads();
}

// ---------------------------------------------------------------- block sums
// part[b] = sum of v[b * kScanBlock .. (b + 1) * kScanBlock) (entries at or past n count as 0).
// No atomics: consecutive groups finish at the same moment, and same-address atomics from all
// of them would serialise the streaming pass.
__device__ __forceinline__ void block_sums_one(const uint32_t* __restrict__ v, long long n, long long b,
                                               unsigned long long* __restrict__ part, unsigned long long* sh) {
  const long long i0 = b * kScanBlock + (long long)threadIdx.x * 4;
  unsigned long long s = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) s += (i0 + j < n) ? v[i0 + j] : 0u;
  const unsigned long long tot = block_sum(s, sh);
  if (threadIdx.x == 0) part[b] = tot;
}

// Block sums of the groups' candidate counts (groups of dense tensors count as zero).
__global__ __launch_bounds__(256) void k_group_sums(Workspace ws) {
  __shared__ unsigned long long sh[4];
  const long long b = blockIdx.x;
  const long long i0 = b * kScanBlock + (long long)threadIdx.x * 4;
  unsigned long long s = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const long long grp = i0 + j;
    if (grp < ws.ngroups) {
      const bool sampled = ws.recs ? (ws.recs[grp].tensor >> 31) != 0u : true;
      const uint32_t c = sampled ? ws.grp_cnt[grp] : 0u;
      if (!sampled) ws.grp_cnt[grp] = 0u;
      s += c;
    }
  }
  const unsigned long long tot = block_sum(s, sh);
  if (threadIdx.x == 0) ws.grp_part[b] = tot;
}

__global__ __launch_bounds__(256) void k_chunk_sums(Workspace ws) {
  __shared__ unsigned long long sh[4];
  const long long n = ws.totals[0] * 4;
  const long long nblocks = (n + kScanBlock - 1) / kScanBlock;
  for (long long b = blockIdx.x; b < nblocks; b += gridDim.x) {
    block_sums_one(ws.ch_gt, n, b, ws.ch_part_gt, sh);
    block_sums_one(ws.ch_eq, n, b, ws.ch_part_eq, sh);
  }
}

// ---------------------------------------------------------------- a threshold inside a huge tie
// A sampled tensor whose candidate list overflows usually does so because the k-th magnitude sits in
// a long run of EQUAL keys (fewer non-zeros than k: the run of zeros; all-equal data; values on a
// coarse grid). Then one counting pass settles the select: if K is that key, c_gt = #(key > K) < k
// and c_gt + #(key == K) >= k, then K is the k-th largest key and k - c_gt of its entries are kept,
// and the three histogram passes over the whole residual are not needed. K is only GUESSED here,
// from the first candidate record of 64 groups spread over the tensor (the smallest key among
// them, if nearly all of them agree); the counts that verify it are exact, and when they do not
// the digit passes run as usual. Single-tensor calls only.
__device__ uint32_t tie_hint_of(const Workspace& ws, const TensorDesc& d) {
  const long long stride = d.ngroups / 64 > 0 ? d.ngroups / 64 : 1;
  uint32_t kmin = kNoTieHint;
  int valid = 0, equal = 0;
  for (int pass = 0; pass < 2; ++pass) {
    for (int i = 0; i < 64; ++i) {
      const long long g = d.group_begin + min((long long)i * stride, (long long)d.ngroups - 1);
      if (ws.grp_cnt[g] == 0u) continue;
      const uint32_t key = ws.slots[g * (int64_t)ws.slot_stride].x & 0x7FFFFFFFu;
      if (pass == 0) {
        kmin = min(kmin, key);
        ++valid;
      } else if (key == kmin) {
        ++equal;
      }
    }
  }
  return (valid >= 8 && equal * 8 >= valid * 7) ? kmin : kNoTieHint;
}

// The counting pass, run in the launch of k_gather (which has nothing to gather for such a tensor):
// a workgroup takes the groups the gather would have given it; per group of 1024 elements - the same
// pieces the dense route's count and emit passes use - the entries above and equal to the hinted
// key, written where k_count would write them, and the workgroup's totals as one pair of partial
// sums (in the group offsets' array, unused on this route; no atomics).
__device__ void tie_spec_count(const Workspace& ws, const float* __restrict__ e, uint32_t hint, int groups_per_wg) {
  __shared__ unsigned long long sh_g[4], sh_e[4];
  const TensorDesc d = ws.desc(0);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long long g0 = (long long)blockIdx.x * groups_per_wg;
  const long long g1 = min((long long)d.ngroups, g0 + groups_per_wg);
  unsigned long long tot_g = 0ull, tot_e = 0ull;
  for (long long lg = g0 + wave; lg < g1; lg += 4) {
    const long long first = max(0ll, lg * (long long)kGroup - d.group_shift);
    const int len = (int)(min((long long)d.n, (lg + 1) * (long long)kGroup - d.group_shift) - first);
    const float* src = e + d.off + first;
    uint32_t gt = 0u, eq = 0u;
    if (len == kChunk && (reinterpret_cast<uintptr_t>(src) & 15u) == 0) {
      f32x4 x[kChunk / 256];
#pragma unroll
      for (int u = 0; u < kChunk / 256; ++u) x[u] = *reinterpret_cast<const f32x4*>(src + u * 256 + lane * 4);
#pragma unroll
      for (int u = 0; u < kChunk / 256; ++u) {
        const uint32_t key[4] = {key_of(x[u].x), key_of(x[u].y), key_of(x[u].z), key_of(x[u].w)};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          gt += key[c] > hint ? 1u : 0u;
          eq += key[c] == hint ? 1u : 0u;
        }
      }
    } else {
      for (int j = lane; j < len; j += 64) {
        const uint32_t key = key_of(src[j]);
        gt += key > hint ? 1u : 0u;
        eq += key == hint ? 1u : 0u;
      }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      gt += __shfl_xor(gt, off);
      eq += __shfl_xor(eq, off);
    }
    if (lane == 0) {
      ws.ch_gt[lg] = gt;  // the sub-chunk numbering of a single tensor is its group numbering
      ws.ch_eq[lg] = eq;
    }
    tot_g += gt;
    tot_e += eq;
  }
  if (g1 == d.ngroups && threadIdx.x < 4) {  // the last chunk's pieces past the tensor's end hold nothing
    const long long lg = d.ngroups + threadIdx.x;
    if (lg < ((d.ngroups + 3) & ~3ll)) {
      ws.ch_gt[lg] = 0u;
      ws.ch_eq[lg] = 0u;
    }
  }
  if (lane == 0) {
    sh_g[wave] = tot_g;
    sh_e[wave] = tot_e;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    ws.grp_off[2 * (long long)blockIdx.x] = (long long)(sh_g[0] + sh_g[1] + sh_g[2] + sh_g[3]);
    ws.grp_off[2 * (long long)blockIdx.x + 1] = (long long)(sh_e[0] + sh_e[1] + sh_e[2] + sh_e[3]);
  }
}

// Whether the hinted key is the threshold: the sums of the counting pass's partials (all 256 threads).
__device__ bool tie_verify(const Workspace& ws, unsigned long long* sh, unsigned long long& c_gt,
                           unsigned long long& c_eq) {
  const long long nwg = (ws.ngroups * ws.gather_team + 255) / 256;  // workgroups of the k_gather launch
  unsigned long long g = 0ull, q = 0ull;
  for (long long i = threadIdx.x; i < nwg; i += 256) {
    g += (unsigned long long)ws.grp_off[2 * i];
    q += (unsigned long long)ws.grp_off[2 * i + 1];
  }
  c_gt = block_sum(g, sh);
  c_eq = block_sum(q, sh);
  const unsigned long long k = (unsigned long long)ws.desc(0).k;
  return c_gt < k && c_gt + c_eq >= k;
}

__device__ __forceinline__ bool tie_hinted(const Workspace& ws) {
  return ws.T == 1 && ws.ts[0].use_cand == 0u && ws.ts[0].tie_hint != kNoTieHint;
}

// ---------------------------------------------------------------- k_group_scan
__global__ __launch_bounds__(256) void k_group_scan(Workspace ws) {
  __shared__ long long lds_out[kScanBlock + 1];
  __shared__ unsigned long long sh[4];
  const int64_t b = blockIdx.x;
  scan_block(ws.grp_cnt, ws.ngroups, ws.grp_part, b, ws.grp_off, lds_out, sh);
  const int64_t lo = b * kScanBlock, hi = lo + kScanBlock;
  for (int t = threadIdx.x; t < ws.T; t += 256) {
    const int64_t gb = ws.desc(t).group_begin;
    if (gb >= lo && gb < hi) ws.tg_base[t] = lds_out[gb - lo];
  }
  if (threadIdx.x == 0 && hi >= ws.ngroups) {
    const long long total = lds_out[min((int64_t)kScanBlock, ws.ngroups - lo)];
    ws.tg_base[ws.T] = total;
    if (ws.T == 1) {
      // a single tensor needs no routing kernel: the block that knows the candidate total decides
      // where the select reads from (what k_route does per tensor when there are several)
      const TensorDesc d = ws.desc(0);
      const bool use = total >= d.k && total <= d.cand_cap;
      const long long vlen = use ? total : d.n;
      ws.ts[0].vlen = vlen;
      ws.ts[0].achunk_begin = 0;
      ws.ts[0].cand_total = total;
      ws.ts[0].use_cand = use ? 1u : 0u;
      ws.ts[0].resolved = 0u;
      ws.ts[0].tie_hint = (!use && total > d.cand_cap) ? tie_hint_of(ws, d) : kNoTieHint;
      ws.totals[0] = (vlen + (use ? 0 : d.group_shift) + kChunkElems - 1) / kChunkElems;
    }
  }
}

// ---------------------------------------------------------------- k_route
// Per tensor: where the select reads from, how long that source is, and its first chunk in
// the call-wide numbering of active chunks (4096 entries each).
__global__ __launch_bounds__(256) void k_route(Workspace ws, int any_sampled) {
  __shared__ unsigned long long sh[4];
  __shared__ long long carry;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int t0 = 0; t0 < ws.T; t0 += 256) {
    const int t = t0 + threadIdx.x;
    long long nch = 0, vlen = 0, M = 0;
    uint32_t use = 0u;
    bool small = false;
    if (t < ws.T) {
      const TensorDesc d = ws.desc(t);
      small = d.small != 0;  // finished by k_finish: no chunks in the grid-wide passes
      vlen = d.n;
      if (d.mode == kSampled && any_sampled && !small) {
        M = ws.tg_base[t + 1] - ws.tg_base[t];
        if (M >= d.k && M <= d.cand_cap) { use = 1u; vlen = M; }
      }
      nch = small ? 0 : (vlen + (use ? 0 : d.group_shift) + kChunkElems - 1) / kChunkElems;
    }
    long long incl = nch;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const long long u = __shfl_up(incl, off);
      if (lane >= off) incl += u;
    }
    __syncthreads();
    if (lane == 63) sh[wave] = (unsigned long long)incl;
    __syncthreads();
    long long x = carry + incl - nch;
    for (int w = 0; w < wave; ++w) x += (long long)sh[w];
    if (t < ws.T) {
      ws.ts[t].achunk_begin = x;
      if (!small) {  // k_finish has written these for its tensors
        ws.ts[t].tie_hint = kNoTieHint;
        ws.ts[t].resolved = 0u;
        ws.ts[t].vlen = vlen;
        ws.ts[t].cand_total = M;
        ws.ts[t].use_cand = use;
      }
    }
    __syncthreads();
    if (threadIdx.x == 255) carry = x + nch;
    __syncthreads();
  }
  if (threadIdx.x == 0) ws.totals[0] = carry;
}

// ---------------------------------------------------------------- k_gather
// TEAM lanes per group copy the group's candidates to their place in the tensor's dense array:
// one lane when a group holds at most one line of records (low density: most groups have one or
// two), 16 lanes with coalesced loads and stores when it holds more. A group with more
// candidates than slots (winners clustered in one stretch of the tensor) is re-read from the
// residual, which holds acc by now, by the whole wavefront: 64 coalesced loads and ballot-ordered
// appends. Only the tensor-wide totals can still send a tensor down the dense route.
template <int TEAM>
__global__ __launch_bounds__(256) void k_gather(Workspace ws, const float* __restrict__ e) {
  if (tie_hinted(ws)) {  // nothing to gather: this launch counts around the hinted tie instead
    tie_spec_count(ws, e, ws.ts[0].tie_hint, 256 / TEAM);
    return;
  }
  const int lane = threadIdx.x & 63;
  const int sub = threadIdx.x % TEAM;  // lane inside the team
  const int64_t grp = ((int64_t)blockIdx.x * 256 + threadIdx.x) / TEAM;
  bool big = false;
  long long dst = 0, first = 0, gbase = 0;
  int glen = 0;
  uint32_t t_lo = 0u;
  if (grp < ws.ngroups) {
    const int t = find_last_le(ws.T, grp, 0, [&](int i) { return (long long)ws.desc(i).group_begin; });
    if (!ws.desc(t).small && ws.ts[t].use_cand != 0u) {
      const TensorDesc d = ws.desc(t);
      const uint32_t cnt = ws.grp_cnt[grp];
      dst = d.cand_begin + (ws.grp_off[grp] - ws.tg_base[t]);
      const long long lg = grp - d.group_begin;
      first = max(0ll, lg * (long long)kGroup - d.group_shift);  // first element of the group in the tensor
      if (cnt > (uint32_t)ws.cap) {
        if (sub == 0) {
          big = true;
          gbase = d.off + first;
          glen = (int)(min((long long)d.n, (lg + 1) * (long long)kGroup - d.group_shift) - first);
          t_lo = ws.ts[t].t_lo;
        }
      } else if (cnt != 0u) {
        const uint2* __restrict__ rec = ws.slots + grp * (int64_t)ws.slot_stride;
        if (TEAM == 1) {
          for (uint32_t j0 = 0; j0 < cnt; j0 += 8) {  // all loads of a round are issued before the stores
            // two records per 128-bit load (a group has 8 or a multiple of 16 slots, 64-byte aligned,
            // and cnt is at most their number: every pair that is read lies inside them)
            uint2 r[8];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              uint4 x = make_uint4(0u, 0u, 0u, 0u);
              if (j0 + 2 * u < cnt) x = reinterpret_cast<const uint4*>(rec + j0)[u];
              r[2 * u] = make_uint2(x.x, x.y);
              r[2 * u + 1] = make_uint2(x.z, x.w);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
              if (j0 + u < cnt) {
                ws.cand_val[dst + j0 + u] = __uint_as_float(r[u].x);
                ws.cand_idx[dst + j0 + u] = first + r[u].y;
              }
            }
          }
        } else {
          for (uint32_t j = sub; j < cnt; j += TEAM) {
            const uint2 r = rec[j];
            ws.cand_val[dst + j] = __uint_as_float(r.x);
            ws.cand_idx[dst + j] = first + r.y;
          }
        }
      }
    }
  }
  uint64_t todo = __ballot(big);
  while (todo) {  // wave-uniform loop over this wavefront's overflowed groups
    const int src = __ffsll((unsigned long long)todo) - 1;
    todo &= todo - 1;
    const long long o_dst = __shfl(dst, src), o_first = __shfl(first, src), o_base = __shfl(gbase, src);
    const int o_len = __shfl(glen, src);
    const uint32_t o_tlo = __shfl(t_lo, src);
    long long w = o_dst;
    for (int j0 = 0; j0 < o_len; j0 += 64) {
      const int j = j0 + lane;
      const float v = j < o_len ? e[o_base + j] : 0.0f;
      const bool c = j < o_len && key_of(v) >= o_tlo;
      const uint64_t m = __ballot(c);
      if (c) {
        const long long pos = w + mbcnt64(m);
        ws.cand_val[pos] = v;
        ws.cand_idx[pos] = o_first + j;
      }
      w += __popcll(m);
    }
  }
}

// ---------------------------------------------------------------- source of the select passes
// A wavefront reads one sub-chunk (1024 entries) of a tensor's select source: the dense
// candidate array, or the residual itself (which holds acc after the streaming pass).
struct SubSrc {
  const float* val;      // values, ascending index order
  const long long* idx;  // element index inside the tensor (null: first + position)
  long long first;
  int len;
};

__device__ __forceinline__ SubSrc sub_source(const Workspace& ws, const TensorDesc& d, const TensorState& st,
                                             long long lchunk, int wave, const float* e) {
  SubSrc s;
  const long long grid_pos = lchunk * kChunkElems + (long long)wave * kChunk;
  if (st.use_cand) {
    s.len = (int)max(0ll, min((long long)kChunk, st.vlen - grid_pos));
    s.first = grid_pos;
    s.val = ws.cand_val + d.cand_begin + grid_pos;
    s.idx = ws.cand_idx + d.cand_begin + grid_pos;
  } else {
    // the residual is cut on the flat buffer's 16-byte grid (as the groups are): only the
    // tensor's first sub-chunk can start unaligned
    const long long pos = max(0ll, grid_pos - d.group_shift);
    const long long end = min((long long)st.vlen, grid_pos + kChunk - d.group_shift);
    s.len = (int)max(0ll, end - pos);
    s.first = pos;
    s.val = e + d.off + pos;
    s.idx = nullptr;
  }
  return s;
}

// ---------------------------------------------------------------- k_hist
__global__ __launch_bounds__(256) void k_hist(Workspace ws, int level, const float* __restrict__ e) {
  __shared__ uint32_t lh[kSelBins];
  if (tie_hinted(ws)) {  // a verified tie at the threshold needs no digit passes
    if (level == 0) {
      __shared__ unsigned long long sh_v[4];
      unsigned long long c_gt, c_eq;
      if (tie_verify(ws, sh_v, c_gt, c_eq)) return;
    } else if (ws.ts[0].resolved) {
      return;
    }
  }
  const long long A = ws.totals[0];
  const long long per = (A + gridDim.x - 1) / gridDim.x;  // one contiguous run of chunks per workgroup
  const long long a_end = min(A, ((long long)blockIdx.x + 1) * per);
  if ((long long)blockIdx.x * per >= a_end) return;  // the grid is sized for the worst case (the dense route)
  for (int b = threadIdx.x; b < kSelBins; b += 256) lh[b] = 0u;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int shift = sel_shift(level);
  const uint32_t mask = (1u << sel_bits(level)) - 1u;
  const int pshift = shift + sel_bits(level);  // bits above this digit must match the prefix
  int cur = -1;
  for (long long a = (long long)blockIdx.x * per; a < a_end; ++a) {
    const int t = find_last_le(ws.T, a, cur < 0 ? 0 : cur, [&](int i) { return ws.ts[i].achunk_begin; });
    if (t != cur) {
      if (cur >= 0) {
        __syncthreads();
        flush_lds_hist<kSelBins>(lh, ws.hist + (int64_t)cur * kSelBins);
        __syncthreads();
      }
      cur = t;
    }
    const TensorDesc d = ws.desc(t);
    const TensorState st = ws.ts[t];
    const SubSrc s = sub_source(ws, d, st, a - st.achunk_begin, wave, e);
    const uint32_t want = (level == 0) ? 0u : (st.prefix >> pshift);
    if (s.len == kChunk && (reinterpret_cast<uintptr_t>(s.val) & 15u) == 0) {
      // a full sub-chunk: four 128-bit loads per lane, all in flight before the first is used
      f32x4 x[kChunk / 256];
#pragma unroll
      for (int u = 0; u < kChunk / 256; ++u) x[u] = *reinterpret_cast<const f32x4*>(s.val + u * 256 + lane * 4);
#pragma unroll
      for (int u = 0; u < kChunk / 256; ++u) {
        const uint32_t key[4] = {key_of(x[u].x), key_of(x[u].y), key_of(x[u].z), key_of(x[u].w)};
#pragma unroll
        for (int c = 0; c < 4; ++c)
          hist_add(lh, level == 0 || (key[c] >> pshift) == want, (key[c] >> shift) & mask);
      }
    } else {
      for (int j0 = 0; j0 < s.len; j0 += 64) {  // uniform trip count: hist_add is a wavefront-wide call
        const int j = j0 + lane;
        const uint32_t key = j < s.len ? key_of(s.val[j]) : 0u;
        hist_add(lh, j < s.len && (level == 0 || (key >> pshift) == want), (key >> shift) & mask);
      }
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
  const TensorDesc d = ws.desc(t);
  if (d.small) return;
  bool resolved = false;
  if (tie_hinted(ws)) {
    if (level == 0) {
      __shared__ unsigned long long sh_v[4];
      unsigned long long c_gt, c_eq;
      resolved = tie_verify(ws, sh_v, c_gt, c_eq);
      if (resolved && threadIdx.x == 0) {  // the hinted key IS the k-th largest: threshold and tie quota
        ws.ts[0].prefix = ws.ts[0].tie_hint;
        ws.ts[0].k_rem = (unsigned long long)d.k - c_gt;
        ws.ts[0].resolved = 1u;
      }
    } else {
      resolved = ws.ts[0].resolved != 0u;
    }
  }
  if (!resolved) {
    unsigned long long* h = ws.hist + (int64_t)t * kSelBins;
    const unsigned long long k_rem = (level == 0) ? (unsigned long long)d.k : ws.ts[t].k_rem;
    uint32_t bin;
    unsigned long long above;
    find_from_top<kSelBins, 256>(h, k_rem, bin, above);
    for (int b = threadIdx.x; b < kSelBins; b += 256) h[b] = 0ull;  // ready for the next digit
    if (threadIdx.x == 0) {
      ws.ts[t].k_rem = k_rem - above;
      const uint32_t p = (level == 0) ? 0u : ws.ts[t].prefix;
      ws.ts[t].prefix = p | (bin << sel_shift(level));
    }
  }
}

// ---------------------------------------------------------------- k_count
__global__ __launch_bounds__(256) void k_count(Workspace ws, const float* __restrict__ e) {
  if (tie_hinted(ws) && ws.ts[0].resolved) return;  // the counting pass around the tie has left these counts
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long long A = ws.totals[0];
  int cur = 0;
  for (long long a = blockIdx.x; a < A; a += gridDim.x) {
    const int t = find_last_le(ws.T, a, cur, [&](int i) { return ws.ts[i].achunk_begin; });
    cur = t;
    const TensorDesc d = ws.desc(t);
    const TensorState st = ws.ts[t];
    const SubSrc s = sub_source(ws, d, st, a - st.achunk_begin, wave, e);
    const uint32_t thr = st.prefix;
    uint32_t gt = 0, eq = 0;
    if (s.len == kChunk && (reinterpret_cast<uintptr_t>(s.val) & 15u) == 0) {
      f32x4 x[kChunk / 256];
#pragma unroll
      for (int u = 0; u < kChunk / 256; ++u) x[u] = *reinterpret_cast<const f32x4*>(s.val + u * 256 + lane * 4);
      uint32_t g4 = 0, e4 = 0;  // per lane; only the sub-chunk's totals are needed here
#pragma unroll
      for (int u = 0; u < kChunk / 256; ++u) {
        const uint32_t key[4] = {key_of(x[u].x), key_of(x[u].y), key_of(x[u].z), key_of(x[u].w)};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          g4 += key[c] > thr ? 1u : 0u;
          e4 += key[c] == thr ? 1u : 0u;
        }
      }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) {
        g4 += __shfl_xor(g4, off);
        e4 += __shfl_xor(e4, off);
      }
      gt = g4;
      eq = e4;
    } else
    for (int j0 = 0; j0 < s.len; j0 += 256) {
      uint32_t key[4];
      bool valid[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int j = j0 + u * 64 + lane;
        valid[u] = j < s.len;
        key[u] = valid[u] ? key_of(s.val[j]) : 0u;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        gt += (uint32_t)__popcll(__ballot(valid[u] && key[u] > thr));
        eq += (uint32_t)__popcll(__ballot(valid[u] && key[u] == thr));
      }
    }
    if (lane == 0) {
      const long long ent = a * 4 + wave;
      ws.ch_gt[ent] = gt;
      ws.ch_eq[ent] = eq;
    }
  }
}

// ---------------------------------------------------------------- k_chunk_scan
__global__ __launch_bounds__(256) void k_chunk_scan(Workspace ws) {
  __shared__ long long lds_out[kScanBlock + 1];
  __shared__ unsigned long long sh[4];
  const long long A = ws.totals[0];
  const long long n = A * 4;
  const long long nblocks = (n + kScanBlock - 1) / kScanBlock;
  for (long long b = blockIdx.x; b < nblocks; b += gridDim.x) {
    const long long lo = b * kScanBlock, hi = lo + kScanBlock;
    scan_block(ws.ch_gt, n, ws.ch_part_gt, b, ws.ch_goff, lds_out, sh);
    for (int t = threadIdx.x; t < ws.T; t += 256) {
      const long long ent = ws.ts[t].achunk_begin * 4;
      if (ent >= lo && ent < hi) ws.tb_g[t] = lds_out[ent - lo];
    }
    __syncthreads();
    scan_block(ws.ch_eq, n, ws.ch_part_eq, b, ws.ch_eoff, lds_out, sh);
    for (int t = threadIdx.x; t < ws.T; t += 256) {
      const long long ent = ws.ts[t].achunk_begin * 4;
      if (ent >= lo && ent < hi) ws.tb_e[t] = lds_out[ent - lo];
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------- k_emit
// Ordered compaction: kept entry number r of a tensor (entries above the threshold, plus the first
// ties in index order up to the quota) goes to position r of the tensor's output, with its value.
//
// Every wavefront works on its own. Piece p (1024 entries) belongs to wavefront p mod (number of
// wavefronts); a wavefront looks at 64 of its pieces at once, one per lane, finds which of them
// keep anything at all, and walks only those. A piece keeps nothing when it has no entry above
// the threshold and its ties are past the quota (or it has none): on the dense route that is
// nearly every piece, since at most k entries are kept. Neighbouring pieces go to different
// wavefronts, so a stretch of pieces that all keep something (the front of a huge tie) is spread.
// The walk is a chain of memory round trips per piece, so the lanes fetch their pieces' offsets
// during the look, and the entries of the next piece are requested before the current one is used.
struct EmitPiece {
  SubSrc s;
  long long G, E;      // kept entries above the threshold / ties before this piece, inside the tensor
  long long out0;      // the tensor's first output position
  long long off;       // the tensor's first element in the flat buffer
  long long quota;
  uint32_t thr;
};

__device__ __forceinline__ long long readlane64(long long v, int l) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, l);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((unsigned long long)v >> 32), l);
  return (long long)(((unsigned long long)hi << 32) | lo);
}

template <typename I>
__global__ __launch_bounds__(256) void k_emit(Workspace ws, const float* __restrict__ e, I* __restrict__ out_idx) {
  constexpr int kIter = kChunk / 64;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const long long N4 = ws.totals[0] * 4;
  const long long gw = (long long)blockIdx.x * 4 + wave, nwv = (long long)gridDim.x * 4;
  for (long long base = gw; base < N4; base += nwv * 64) {
    bool need = false;
    long long my_g = 0, my_e = 0;
    int my_t = 0;
    {
      const long long ent_l = base + lane * nwv;
      if (ent_l < N4) {
        const uint32_t gt = ws.ch_gt[ent_l], eq = ws.ch_eq[ent_l];
        if ((gt | eq) != 0u) {
          my_t = find_last_le(ws.T, ent_l >> 2, 0, [&](int i) { return ws.ts[i].achunk_begin; });
          my_e = ws.ch_eoff[ent_l] - ws.tb_e[my_t];
          need = gt != 0u || my_e < (long long)ws.ts[my_t].k_rem;
          if (need) my_g = ws.ch_goff[ent_l] - ws.tb_g[my_t];
        }
      }
    }
    uint64_t todo = __ballot(need);
    if (todo == 0ull) continue;
    // the piece of lane `bit`: where its entries are, and the request for them
    auto open = [&](int bit, EmitPiece& p, float (&vals)[kIter]) {
      const long long ent = base + bit * nwv, a = ent >> 2;
      const int t = __builtin_amdgcn_readlane(my_t, bit);
      const TensorDesc d = ws.desc(t);
      const TensorState st = ws.ts[t];
      p.s = sub_source(ws, d, st, a - st.achunk_begin, (int)(ent & 3), e);
      p.G = readlane64(my_g, bit);
      p.E = readlane64(my_e, bit);
      p.out0 = d.kprefix;
      p.off = d.off;
      p.quota = (long long)st.k_rem;
      p.thr = st.prefix;
#pragma unroll
      for (int u = 0; u < kIter; ++u) {
        const int j = u * 64 + lane;
        vals[u] = j < p.s.len ? p.s.val[j] : 0.0f;
      }
    };
    EmitPiece cur, nxt;
    float vals[kIter], nvals[kIter];
    open(__builtin_amdgcn_readfirstlane(__ffsll((unsigned long long)todo) - 1), cur, vals);
    todo &= todo - 1;
    while (true) {
      const bool more = todo != 0ull;
      if (more) {
        open(__builtin_amdgcn_readfirstlane(__ffsll((unsigned long long)todo) - 1), nxt, nvals);
        todo &= todo - 1;
      }
      long long idxs[kIter];
#pragma unroll
      for (int u = 0; u < kIter; ++u) {
        const int j = u * 64 + lane;
        idxs[u] = (cur.s.idx && j < cur.s.len) ? cur.s.idx[j] : (cur.s.first + j);
      }
      long long G = cur.G, E = cur.E;
#pragma unroll
      for (int u = 0; u < kIter; ++u) {
        const int j0 = u * 64;
        if (j0 >= cur.s.len) continue;  // uniform over the wavefront
        const bool valid = j0 + lane < cur.s.len;
        const float v = vals[u];
        const uint32_t key = key_of(v);
        const bool isgt = valid && key > cur.thr, iseq = valid && key == cur.thr;
        const uint64_t mg = __ballot(isgt), me = __ballot(iseq);
        if ((mg | me) == 0ull) continue;  // nothing at or above the threshold in these 64 entries
        const long long grank = G + mbcnt64(mg), erank = E + mbcnt64(me);
        if (isgt || (iseq && erank < cur.quota)) {
          const long long pos = cur.out0 + grank + (erank < cur.quota ? erank : cur.quota);
          out_idx[pos] = (I)(cur.off + idxs[u]);
          ws.kept_val[pos] = v;
        }
        G += __popcll(mg);
        E += __popcll(me);
      }
      if (!more) break;
      cur = nxt;
#pragma unroll
      for (int u = 0; u < kIter; ++u) vals[u] = nvals[u];
    }
  }
}

// ---------------------------------------------------------------- k_quant
// Per-block int8 code of the kept values (Eq. 9) and the residual at the kept positions,
// e' = acc - fl32(q * s) (Eq. 11). The kept entries of all tensors form one array of sum(k)
// positions, cut into blocks tensor by tensor. A workgroup codes its own kQuantSpan positions; the
// largest magnitude of every block that reaches into them it finds itself, by reading those blocks
// whole (wavefront maximum, then one LDS atomic; a maximum does not depend on the order).
// Neighbouring workgroups read the same block again, out of the cache, which is little beside the
// scattered residual stores. No block maximum ever goes through memory.
// Blocks longer than kQuantSharedBlock would make that re-reading the main cost: then a workgroup
// owns the blocks that START inside its positions instead and codes all of their entries.
constexpr int kQuantSharedBlock = 4096;
constexpr int kQuantSpan = 1024;  // kept positions per workgroup

constexpr int kQuantLdsTensors = 1024;  // the tensors' first kept positions are staged in LDS up to this many

// Start of the first block at or after kept position x (x itself if a block starts there), given
// the tensor t that holds x. kp(i): first kept position of tensor i.
template <typename KP>
__device__ __forceinline__ long long next_block_start(const Workspace& ws, KP kp, int t, long long x, FastDiv bdiv,
                                                      int32_t block) {
  const long long k0 = kp(t), rel = x - k0;  // rel < k < 2^32
  const uint32_t rb = fast_div((uint32_t)rel, bdiv);
  if ((long long)rb * block == rel) return x;
  return k0 + min((long long)ws.desc(t).k, ((long long)rb + 1) * block);
}

template <typename I>
__global__ __launch_bounds__(256) void k_quant(Workspace ws, float* __restrict__ e,
                                               const I* __restrict__ idx, int8_t* __restrict__ q,
                                               float* __restrict__ scales, int32_t block, FastDiv bdiv, long long ktotal) {
  // blocks that reach into the span: one may start at each position, one more may have started before
  __shared__ uint32_t amax[kQuantSpan + 1];
  // Which tensor a kept position belongs to is a binary search over the tensors' first positions:
  // out of LDS, not a chain of dependent loads from memory, when there are several tensors. Their
  // first blocks and their routes are staged with them.
  __shared__ uint32_t s_kp[kQuantLdsTensors], s_sp[kQuantLdsTensors];
  __shared__ uint8_t s_small[kQuantLdsTensors];
  const int tid = threadIdx.x, lane = tid & 63;
  const bool staged = ws.T > 1 && ws.T <= kQuantLdsTensors;  // uniform over the grid
  if (staged) {
    for (int t = tid; t < ws.T; t += 256) {
      s_kp[t] = (uint32_t)ws.desc(t).kprefix;  // both below 2^32
      s_sp[t] = (uint32_t)ws.desc(t).sprefix;
      s_small[t] = ws.desc(t).small ? 1 : 0;
    }
    __syncthreads();
  }
  auto kp = [&](int i) -> long long { return staged ? (long long)s_kp[i] : (long long)ws.desc(i).kprefix; };
  auto sp = [&](int i) -> long long { return staged ? (long long)s_sp[i] : (long long)ws.desc(i).sprefix; };
  auto small = [&](int i) -> bool { return staged ? s_small[i] != 0 : ws.desc(i).small != 0; };
  const long long lo = (long long)blockIdx.x * kQuantSpan, hi = min(ktotal, lo + kQuantSpan);
  const bool own = block <= kQuantSharedBlock;  // the workgroup codes its own positions
  constexpr int kU = kQuantSpan / 256;  // strides of 256 positions whose loads are in flight together
  // its own entries are asked for before anything else: nothing below depends on them until the codes
  float v_own[kU];
  I at_own[kU];
#pragma unroll
  for (int u = 0; u < kU; ++u) {
    const long long j = lo + u * 256 + tid;
    v_own[u] = (own && j < hi) ? ws.kept_val[j] : 0.0f;
    at_own[u] = (own && j < hi) ? idx[j] : (I)0;
  }
  const int t_lo = find_last_le(ws.T, lo, 0, kp);  // one search; the tensors after it by hint
  const int t_hi = hi < ktotal ? find_last_le(ws.T, hi, t_lo, kp) : ws.T - 1;
  const long long e_hi = hi < ktotal ? next_block_start(ws, kp, t_hi, hi, bdiv, block) : ktotal;
  long long m_lo, m_hi, c_lo, c_hi;  // positions read for the maxima, positions coded
  if (own) {
    m_lo = kp(t_lo) + (long long)fast_div((uint32_t)(lo - kp(t_lo)), bdiv) * block;  // start of the block that holds lo
    m_hi = e_hi;
    c_lo = lo;
    c_hi = hi;
  } else {
    m_lo = c_lo = next_block_start(ws, kp, t_lo, lo, bdiv, block);
    m_hi = c_hi = e_hi;
    if (c_lo >= c_hi) return;  // no block starts here (uniform over the workgroup)
  }
  const int t_s = find_last_le(ws.T, m_lo, t_lo, kp);
  // a span that only small tensors reach into has nothing to do here (they are coded by k_finish):
  // with many small tensors that is most workgroups, and their per-position searches were the
  // longest thing in the launch
  {
    int general = 0;
    for (int t = t_s + tid; t <= t_hi; t += 256) general |= small(t) ? 0 : 1;
    if (__syncthreads_or(general) == 0) return;
  }
  const long long blk_s = sp(t_s) + fast_div((uint32_t)(m_lo - kp(t_s)), bdiv);
  for (int b = tid; b < kQuantSpan + 1; b += 256) amax[b] = 0u;
  __syncthreads();
  constexpr int kM = 8;  // the same for the maxima: a block before and a block after the span
  for (long long j0 = m_lo; j0 < m_hi; j0 += 256 * kM) {  // uniform trip count
    bool on[kM];
    uint32_t bl[kM];
    float v[kM];
#pragma unroll
    for (int u = 0; u < kM; ++u) {
      const long long j = j0 + u * 256 + tid;
      on[u] = j < m_hi;
      bl[u] = 0u;
      v[u] = 0.0f;
      if (on[u]) {
        const int t = find_last_le_in(t_s, t_hi, j, kp);
        on[u] = !small(t);  // small tensors are coded by k_finish
        bl[u] = (uint32_t)(sp(t) - blk_s) + fast_div((uint32_t)(j - kp(t)), bdiv);
        if (on[u]) v[u] = ws.kept_val[j];
      }
    }
#pragma unroll
    for (int u = 0; u < kM; ++u) {
      const uint32_t key = key_of(v[u]);
      // nearly always the wavefront's 64 consecutive entries lie in one block: one atomic then
      const uint64_t act = __ballot(on[u]);
      if (act == 0ull) continue;
      const uint32_t bl0 = (uint32_t)__builtin_amdgcn_readlane((int)bl[u], __ffsll((unsigned long long)act) - 1);
      if (__ballot(on[u] && bl[u] != bl0) == 0ull) {
        uint32_t m = on[u] ? key : 0u;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off));
        if (lane == 0) atomicMax(&amax[bl0], m);
      } else if (on[u]) {
        atomicMax(&amax[bl[u]], key);
      }
    }
  }
  __syncthreads();
  for (long long j0 = c_lo; j0 < c_hi; j0 += 256 * kU) {
    bool on[kU];
    uint32_t rel[kU], rblk[kU];
    long long blk[kU];
    float v[kU];
    I at[kU];
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const long long j = j0 + u * 256 + tid;
      on[u] = j < c_hi;
      rel[u] = rblk[u] = 0u;
      blk[u] = blk_s;
      v[u] = 0.0f;
      at[u] = (I)0;
      if (on[u]) {
        const int t = find_last_le_in(t_s, t_hi, j, kp);
        on[u] = !small(t);
        rel[u] = (uint32_t)(j - kp(t));  // < k < 2^32
        rblk[u] = fast_div(rel[u], bdiv);
        blk[u] = sp(t) + rblk[u];
        if (on[u]) {
          v[u] = own ? v_own[u] : ws.kept_val[j];  // own: one batch, j = lo + u * 256 + tid
          at[u] = own ? at_own[u] : idx[j];
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      if (!on[u]) continue;
      const long long j = j0 + u * 256 + tid;
      const uint32_t akey = amax[blk[u] - blk_s];
      const bool finite = akey < 0x7F800000u;
      float s = __fdiv_rn(__uint_as_float(akey), 127.0f);
      if (!finite || !(s >= 1.17549435e-38f)) s = 0.0f;
      if (rel[u] == rblk[u] * (uint32_t)block) {
        scales[blk[u]] = s;
        if (!finite) ws.flags[0] = 1u;
      }
      int code = 0;
      if (s != 0.0f) {
        float r = rintf(__fdiv_rn(v[u], s));
        r = fminf(fmaxf(r, -127.0f), 127.0f);
        code = (int)r;
      }
      q[j] = (int8_t)code;
      if (finite) e[(int64_t)at[u]] = __fsub_rn(v[u], __fmul_rn((float)code, s));
    }
  }
}

// ---------------------------------------------------------------- k_quant_sign
// The 1-bit code of Eq. 10: one workgroup per block of kept entries. The block's l1 norm is
// accumulated in fp64 over the balanced binary tree a[i] += a[i + stride], stride = P/2 .. 1, on the
// entries padded with zeros to a power of two P (levels with stride >= 256 stay inside a thread's
// registers, the rest goes through LDS; padding with +0 is exact, so P = max(256, pow2(len)) gives
// the same sum as pow2(len)). s = (float)(sum / len); bits are packed through wavefront ballots.
constexpr int kSignMaxPerThread = 32;  // block <= 8192
template <typename I>
__global__ __launch_bounds__(256) void k_quant_sign(Workspace ws, float* __restrict__ e,
                                                    const I* __restrict__ idx, uint8_t* __restrict__ q,
                                                    float* __restrict__ scales, int32_t block) {
  __shared__ double sh[256];
  const int64_t gb = blockIdx.x;
  const int t = find_last_le(ws.T, gb, 0, [&](int i) { return (long long)ws.desc(i).sprefix; });
  const TensorDesc d = ws.desc(t);
  const int64_t lb = gb - d.sprefix;
  const int64_t j0 = d.kprefix + lb * block;
  const int len = (int)min((int64_t)block, d.k - lb * block);
  int per = 1;  // entries per thread: P / 256
  while (per * 256 < len) per <<= 1;
  double r[kSignMaxPerThread];
#pragma unroll
  for (int m = 0; m < kSignMaxPerThread; ++m) {
    const int i = threadIdx.x + m * 256;
    r[m] = (m < per && i < len) ? fabs((double)ws.kept_val[j0 + i]) : 0.0;
  }
#pragma unroll
  for (int half = kSignMaxPerThread / 2; half >= 1; half >>= 1) {  // stride = half * 256
    if (half < per) {
#pragma unroll
      for (int m = 0; m < kSignMaxPerThread / 2; ++m)
        if (m < half) r[m] = r[m] + r[m + half];
    }
  }
  sh[threadIdx.x] = r[0];
  __syncthreads();
  for (int stride = 128; stride >= 1; stride >>= 1) {
    if ((int)threadIdx.x < stride) sh[threadIdx.x] = sh[threadIdx.x] + sh[threadIdx.x + stride];
    __syncthreads();
  }
  // an entry that is not finite makes the fp64 sum infinite or NaN; finite entries cannot (2^13 * 2^128)
  const bool finite = sh[0] < (double)INFINITY;
  float s = (float)(sh[0] / (double)len);
  if (!finite || !(s >= 1.17549435e-38f)) s = 0.0f;
  if (threadIdx.x == 0) {
    scales[gb] = s;
    if (!finite) ws.flags[0] = 1u;
  }
  // this block's bytes: blocks before it in the tensor are full
  uint8_t* qb = q + d.qprefix + lb * ((block + 7) / 8);
  const int lane = threadIdx.x & 63;
  for (int i0 = (threadIdx.x >> 6) * 64; i0 < len; i0 += 256) {  // i0 is wave-uniform
    const int i = i0 + lane;
    const bool valid = i < len;
    const float v = valid ? ws.kept_val[j0 + i] : 0.0f;
    const bool plus = valid && v >= 0.0f;
    const uint64_t m = __ballot(plus);
    if (lane < 8 && i0 + lane * 8 < len) qb[i0 / 8 + lane] = (uint8_t)(finite ? (m >> (8 * lane)) & 0xFFull : 0ull);
    if (valid && finite) e[(int64_t)idx[j0 + i]] = __fsub_rn(v, plus ? s : -s);
  }
}

// ---------------------------------------------------------------- k_finish
// One workgroup of 1024 threads finishes one SMALL tensor after the streaming pass: what the chain
// k_group_sums .. k_quant does with a dozen grid-wide launches is done here with workgroup
// barriers in between. Same arithmetic, same order, same bits:
//   1. prefix sum of the tensor's group counts (sampled tensors)
//   2. the select source in ascending index order: the candidates, packed from the groups' slots (a
//      group with more candidates than slots is re-read from the residual); or, with too few or
//      too many candidates and for tensors selected from their residual by plan, the residual
//      itself. A source of up to kFinishLds entries is held in LDS (value bits and index), a longer
//      one stays in memory (candidates: in the tensor's region of the candidate arrays).
//   3. exact radix select (three digits, LDS histogram) of the k-th largest key and the tie quota
//   4. ordered emit: kept entries compacted in place (LDS), or written to the output (memory)
//   5. per block of kept entries: amax (LDS), scale, int8 codes, residual at the kept positions
//      (with the sign code there is no step 5: the kept values go out and k_quant_sign follows)
constexpr int kFinishLds = 16384;     // entries of the LDS-resident source (128 KB)
constexpr int kFinishMaxGroups = 4096;
constexpr int kFinishAmaxWindow = 4096;

template <typename I>
__global__ __launch_bounds__(kFinishThreads) void k_finish(Workspace ws, float* __restrict__ e,
                                                            I* __restrict__ out_idx, int8_t* __restrict__ q,
                                                            float* __restrict__ scales, int32_t block, int codec) {
  constexpr int NT = kFinishThreads, NW = NT / 64;
  const int t = blockIdx.x;
  const TensorDesc d = ws.desc(t);
  if (!d.small) return;
  __shared__ uint32_t lk[kFinishLds];  // value bits of the source / of the kept entries
  __shared__ uint32_t li[kFinishLds];  // element index inside the tensor
  // one region used three times: group offsets (steps 1-2), select histogram (3), block maxima (5)
  __shared__ uint32_t scratch[kFinishMaxGroups + 1];
  static_assert(kSelBins <= kFinishMaxGroups + 1 && kFinishAmaxWindow <= kFinishMaxGroups + 1, "scratch too small");
  uint32_t* goff = scratch;
  uint32_t* lh = scratch;
  uint32_t* amax = scratch;
  __shared__ unsigned long long s_red[NW];
  __shared__ uint32_t s_flag;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // the source when it stays in memory
  const float* gval = e + d.off;
  const long long* gidx = nullptr;
  long long len = d.n;
  bool in_lds = false;
  uint32_t use_cand = 0u;
  long long M = 0;
  if (d.mode == kSampled) {
    // ---- 1. group counts -> offsets (GPT consecutive groups per thread)
    constexpr int GPT = kFinishMaxGroups / NT;
    const int ng = (int)d.ngroups;
    uint32_t c[GPT];
    uint32_t mine = 0u;
#pragma unroll
    for (int j = 0; j < GPT; ++j) {
      const int g = tid * GPT + j;
      c[j] = g < ng ? ws.grp_cnt[d.group_begin + g] : 0u;
      mine += c[j];
    }
    uint32_t incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t u = __shfl_up(incl, off);
      if (lane >= off) incl += u;
    }
    if (lane == 63) s_red[wave] = incl;
    if (tid == 0) s_flag = 0u;
    __syncthreads();
    uint32_t x = incl - mine;
    unsigned long long total = 0ull;
    for (int w = 0; w < NW; ++w) {
      if (w < wave) x += (uint32_t)s_red[w];
      total += s_red[w];
    }
    M = (long long)total;
#pragma unroll
    for (int j = 0; j < GPT; ++j) {
      goff[tid * GPT + j] = x;
      x += c[j];
    }
    if (tid == NT - 1) goff[kFinishMaxGroups] = x;
    use_cand = (M >= d.k && M <= d.cand_cap) ? 1u : 0u;
    if (use_cand) {
      // ---- 2. pack the candidates: one thread per group; the loads of a round are issued together
      in_lds = M <= kFinishLds;
      const uint32_t t_lo = ws.ts[t].t_lo;
      float* cv = ws.cand_val + d.cand_begin;
      long long* ci = ws.cand_idx + d.cand_begin;
      bool any_big = false;
      __syncthreads();  // goff is complete
      // groups are dealt out round robin here (the scan above had four neighbours per thread), so
      // that a tensor with few groups still keeps every thread busy with one group
#pragma unroll 1
      for (int g = tid; g < ng; g += NT) {
        const uint32_t dst = goff[g];
        const uint32_t cnt = goff[g + 1] - dst;
        if (cnt == 0u) continue;
        if (cnt > (uint32_t)ws.cap) { any_big = true; continue; }
        const long long first = max(0ll, (long long)g * kGroup - d.group_shift);
        const uint2* __restrict__ rec = ws.slots + (d.group_begin + g) * (int64_t)ws.slot_stride;
        for (uint32_t j0 = 0; j0 < cnt; j0 += 8) {
          uint2 r[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) r[u] = (j0 + u < cnt) ? rec[j0 + u] : make_uint2(0u, 0u);
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            if (j0 + u < cnt) {
              if (in_lds) {
                lk[dst + j0 + u] = r[u].x;
                li[dst + j0 + u] = (uint32_t)(first + r[u].y);
              } else {
                cv[dst + j0 + u] = __uint_as_float(r[u].x);
                ci[dst + j0 + u] = first + r[u].y;
              }
            }
          }
        }
      }
      if (any_big) s_flag = 1u;
      __syncthreads();
      if (s_flag) {
        // groups with more candidates than slots: a wavefront re-reads the group from the residual
        // (it holds acc by now) and appends with ballot-ordered ranks
        for (int g = wave; g < ng; g += NW) {
          const uint32_t cnt_g = goff[g + 1] - goff[g];  // goff has an entry past the last group
          if (cnt_g <= (uint32_t)ws.cap) continue;       // uniform over the wavefront
          const long long first = max(0ll, (long long)g * kGroup - d.group_shift);
          const int glen = (int)(min((long long)d.n, (long long)(g + 1) * kGroup - d.group_shift) - first);
          long long w = goff[g];
          for (int j0 = 0; j0 < glen; j0 += 64) {
            const int j = j0 + lane;
            const float v = j < glen ? e[d.off + first + j] : 0.0f;
            const bool cnd = j < glen && key_of(v) >= t_lo;
            const uint64_t m = __ballot(cnd);
            if (cnd) {
              const long long pos = w + mbcnt64(m);
              if (in_lds) {
                lk[pos] = __float_as_uint(v);
                li[pos] = (uint32_t)(first + j);
              } else {
                cv[pos] = v;
                ci[pos] = first + j;
              }
            }
            w += __popcll(m);
          }
        }
      }
      gval = cv;
      gidx = ci;
      len = M;
    }
    __syncthreads();  // the packed candidates are visible to the whole workgroup; goff is free
  }
  if (!use_cand && len <= kFinishLds) {  // a short residual is held in LDS too
    in_lds = true;
    for (int i = tid; i < (int)len; i += NT) {
      lk[i] = __float_as_uint(gval[i]);
      li[i] = (uint32_t)i;
    }
    __syncthreads();
  }
  if (tid == 0) {  // what gc_last_stats reports
    ws.ts[t].cand_total = M;
    ws.ts[t].use_cand = use_cand;
    ws.ts[t].vlen = len;
  }

  // ---- 3. exact select: T = k-th largest key, quota = how many entries equal to T are kept.
  // A radix select on key - kmin (order preserving), its digits laid over the range the keys really
  // span: the keys of a candidate list share their top bits, and digits cut from the full 31 bits
  // would pile them into a few bins of the first histogram (LDS atomics on one address run one
  // after the other). With the range [kmin, kmax] cut into at most 2048 bins the first digit
  // spreads them, and the later digits only see the few keys of one bin.
  uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
  for (long long i = tid; i < len; i += NT) {
    const uint32_t key = (in_lds ? lk[i] : __float_as_uint(gval[i])) & 0x7FFFFFFFu;
    kmin = min(kmin, key);
    kmax = max(kmax, key);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, off));
    kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, off));
  }
  if (lane == 0) s_red[wave] = ((unsigned long long)kmax << 32) | kmin;
  __syncthreads();
  for (int w = 0; w < NW; ++w) {
    kmin = min(kmin, (uint32_t)s_red[w]);
    kmax = max(kmax, (uint32_t)(s_red[w] >> 32));
  }
  int shift = 0;  // low bits below the current digit
  while (((kmax - kmin) >> shift) >= (uint32_t)kSelBins) ++shift;
  uint32_t prefix = 0u;  // resolved high part of T - kmin (bits above the current digit)
  int pshift = 32;       // bits of (key - kmin) at or above pshift must match the prefix
  unsigned long long k_rem = (unsigned long long)d.k;
  for (;;) {
    for (int b = tid; b < kSelBins; b += NT) lh[b] = 0u;
    __syncthreads();
    for (long long i0 = 0; i0 < len; i0 += NT) {
      const long long i = i0 + tid;
      const bool valid = i < len;
      const uint32_t rel = valid ? (((in_lds ? lk[i] : __float_as_uint(gval[i])) & 0x7FFFFFFFu) - kmin) : 0u;
      const bool match = pshift >= 32 || (rel >> pshift) == (prefix >> pshift);
      hist_add(lh, valid && match, (rel >> shift) & (uint32_t)(kSelBins - 1));
    }
    __syncthreads();
    uint32_t bin;
    unsigned long long above;
    find_from_top<kSelBins, NT>(lh, k_rem, bin, above);
    k_rem -= above;
    prefix |= bin << shift;
    if (shift == 0) break;
    pshift = shift;
    shift = shift > 11 ? shift - 11 : 0;
  }
  prefix += kmin;
  const uint32_t thr = prefix;
  const long long quota = (long long)k_rem;

  // ---- 4. ordered emit, four tiles of 1024 entries per pair of barriers
  __shared__ uint32_t s_wg4[4][NW], s_we4[4][NW];
  long long G = 0, E = 0;  // entries above / equal to the threshold before the current tiles
  for (long long i0 = 0; i0 < len; i0 += 4 * NT) {
    uint32_t vb[4], ib[4];
    long long ig[4];
    bool isgt[4], iseq[4];
    uint64_t mg[4], me[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const long long i = i0 + u * NT + tid;
      const bool valid = i < len;
      vb[u] = 0u; ib[u] = 0u; ig[u] = 0;
      if (valid) {
        if (in_lds) { vb[u] = lk[i]; ib[u] = li[i]; }
        else { vb[u] = __float_as_uint(gval[i]); ig[u] = gidx ? gidx[i] : i; }
      }
      const uint32_t key = vb[u] & 0x7FFFFFFFu;
      isgt[u] = valid && key > thr;
      iseq[u] = valid && key == thr;
      mg[u] = __ballot(isgt[u]);
      me[u] = __ballot(iseq[u]);
      if (lane == 0) {
        s_wg4[u][wave] = (uint32_t)__popcll(mg[u]);
        s_we4[u][wave] = (uint32_t)__popcll(me[u]);
      }
    }
    __syncthreads();  // every entry of these tiles is in registers: their LDS slots may be overwritten
    long long gt_all = 0, eq_all = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      // lanes 0..15 hold the 16 wavefronts' counts of tile u; an inclusive scan over them gives
      // this wavefront's base (exclusive) and the tile's totals
      uint32_t cg = lane < NW ? s_wg4[u][lane] : 0u, ce = lane < NW ? s_we4[u][lane] : 0u;
      uint32_t sg = cg, se = ce;
#pragma unroll
      for (int off = 1; off < NW; off <<= 1) {
        const uint32_t ug = __shfl_up(sg, off), ue = __shfl_up(se, off);
        if (lane >= off) { sg += ug; se += ue; }
      }
      const long long gb = G + gt_all + (long long)(uint32_t)__builtin_amdgcn_readlane((int)(sg - cg), wave);
      const long long eb = E + eq_all + (long long)(uint32_t)__builtin_amdgcn_readlane((int)(se - ce), wave);
      gt_all += (uint32_t)__builtin_amdgcn_readlane((int)sg, NW - 1);
      eq_all += (uint32_t)__builtin_amdgcn_readlane((int)se, NW - 1);
      const long long grank = gb + mbcnt64(mg[u]), erank = eb + mbcnt64(me[u]);
      if (isgt[u] || (iseq[u] && erank < quota)) {
        const long long rel = grank + (erank < quota ? erank : quota);  // <= i: compaction moves entries down only
        if (in_lds) {
          lk[rel] = vb[u];
          li[rel] = ib[u];
        } else {
          out_idx[d.kprefix + rel] = (I)(d.off + ig[u]);
          ws.kept_val[d.kprefix + rel] = __uint_as_float(vb[u]);
        }
      }
    }
    G += gt_all;
    E += eq_all;
    __syncthreads();  // the counts are rewritten by the next round
  }
  if (in_lds) {  // the kept entries now are lk / li [0, k): indices (and, for k_quant_sign, values) go out
    for (int j = tid; j < (int)d.k; j += NT) {
      out_idx[d.kprefix + j] = (I)(d.off + (long long)li[j]);
      if (codec != 0) ws.kept_val[d.kprefix + j] = __uint_as_float(lk[j]);
    }
  }

  // ---- 5. blocks of kept entries: amax, scale, code, residual (windows of kFinishAmaxWindow blocks)
  if (codec != 0) return;  // uniform over the workgroup
  const long long nblk = (d.k + block - 1) / block;
  for (long long b0 = 0; b0 < nblk; b0 += kFinishAmaxWindow) {
    const long long b1 = min(nblk, b0 + (long long)kFinishAmaxWindow);
    for (int b = tid; b < (int)(b1 - b0); b += NT) amax[b] = 0u;
    __syncthreads();
    const long long j_begin = b0 * block, j_end = min((long long)d.k, b1 * block);
    for (long long j0 = j_begin; j0 < j_end; j0 += NT) {
      const long long j = j0 + tid;
      const bool on = j < j_end;
      uint32_t kb = 0u, bl = 0u;
      if (on) {
        kb = (in_lds ? lk[j] : __float_as_uint(ws.kept_val[d.kprefix + j])) & 0x7FFFFFFFu;
        bl = (uint32_t)j / (uint32_t)block - (uint32_t)b0;
      }
      // nearly always the wavefront's 64 consecutive entries lie in one block: one atomic then
      const uint64_t act = __ballot(on);
      const uint32_t bl0 = (uint32_t)__builtin_amdgcn_readlane((int)bl, act ? __ffsll((unsigned long long)act) - 1 : 0);
      if (__ballot(on && bl != bl0) == 0ull) {
        uint32_t m = kb;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off));
        if (lane == 0 && act) atomicMax(&amax[bl0], m);
      } else if (on) {
        atomicMax(&amax[bl], kb);
      }
    }
    __syncthreads();
    for (int b = tid; b < (int)(b1 - b0); b += NT) {
      const uint32_t akey = amax[b];
      const bool finite = akey < 0x7F800000u;
      float sc = __fdiv_rn(__uint_as_float(akey), 127.0f);
      if (!finite || !(sc >= 1.17549435e-38f)) sc = 0.0f;
      scales[d.sprefix + b0 + b] = sc;
      if (!finite) ws.flags[0] = 1u;
    }
    {
      for (long long j0 = j_begin; j0 < j_end; j0 += NT) {
        const long long j = j0 + tid;
        if (j >= j_end) continue;
        const uint32_t akey = amax[(uint32_t)j / (uint32_t)block - (uint32_t)b0];
        const bool finite = akey < 0x7F800000u;
        float sc = __fdiv_rn(__uint_as_float(akey), 127.0f);
        if (!finite || !(sc >= 1.17549435e-38f)) sc = 0.0f;
        const float v = in_lds ? __uint_as_float(lk[j]) : ws.kept_val[d.kprefix + j];
        const long long pos = in_lds ? d.off + (long long)li[j] : (long long)out_idx[d.kprefix + j];
        int code = 0;
        if (sc != 0.0f) {
          float r = rintf(__fdiv_rn(v, sc));
          r = fminf(fmaxf(r, -127.0f), 127.0f);
          code = (int)r;
        }
        q[d.kprefix + j] = (int8_t)code;
        if (finite) e[pos] = __fsub_rn(v, __fmul_rn((float)code, sc));
      }
    }
    __syncthreads();  // amax is rewritten by the next window
  }
}

inline int clamp_grid(int64_t want, int64_t cap) { return (int)(want < 1 ? 1 : (want > cap ? cap : want)); }

}  // namespace

void launch_sample(const Workspace& ws, const void* g, int dtype, const float* e, hipStream_t s) {
  // every workgroup clears and flushes an 8192-bin histogram: 1024 workgroups measured best (256: the
  // per-workgroup chain of loads gets long; 8192: the flushes dominate)
  const dim3 grid(clamp_grid((ws.nsgran + 3) / 4, 1024));
  if (dtype == 0)
    hipLaunchKernelGGL(k_sample<float>, grid, dim3(256), 0, s, ws, (const float*)g, e);
  else
    hipLaunchKernelGGL(k_sample<uint16_t>, grid, dim3(256), 0, s, ws, (const uint16_t*)g, e);
}

void launch_sample_thresh(const Workspace& ws, hipStream_t s) {
  hipLaunchKernelGGL(k_sample_thresh, dim3(ws.T), dim3(256), 0, s, ws);
}

void launch_main(const Workspace& ws, const void* g, int dtype, float* e, hipStream_t s) {
  const dim3 grid((unsigned)xcd_run_grid(ws.ngroups));
  const size_t pad = (size_t)std::max<int64_t>(ws.main_lds_pad, (int64_t)ws.cap * 8);
  const long long n_single = ws.recs ? 0 : ws.n_single;
  const int sampled_single = ws.nsgran > 0 ? 1 : 0;
  if (dtype == 0)
    hipLaunchKernelGGL(k_main<float>, grid, dim3(256), pad, s, ws, (const float*)g, e, ws.recs, n_single,
                       sampled_single);
  else
    hipLaunchKernelGGL(k_main<uint16_t>, grid, dim3(256), pad, s, ws, (const uint16_t*)g, e, ws.recs,
                       n_single, sampled_single);
}

void launch_group_sums(const Workspace& ws, hipStream_t s) {
  hipLaunchKernelGGL(k_group_sums, dim3((unsigned)((ws.ngroups + kScanBlock - 1) / kScanBlock)), dim3(256), 0, s, ws);
}

void launch_chunk_sums(const Workspace& ws, hipStream_t s) {
  const int64_t blocks = ((int64_t)ws.max_chunk_wgs * 4 + kScanBlock - 1) / kScanBlock;
  hipLaunchKernelGGL(k_chunk_sums, dim3(clamp_grid(blocks, 512)), dim3(256), 0, s, ws);
}

void launch_group_scan(const Workspace& ws, hipStream_t s) {
  hipLaunchKernelGGL(k_group_scan, dim3((unsigned)((ws.ngroups + kScanBlock - 1) / kScanBlock)), dim3(256), 0, s, ws);
}

void launch_route(const Workspace& ws, hipStream_t s) {
  hipLaunchKernelGGL(k_route, dim3(1), dim3(256), 0, s, ws, ws.nsgran > 0 ? 1 : 0);
}

void launch_gather(const Workspace& ws, const float* e, hipStream_t s) {
  const int team = ws.gather_team;  // chosen by the plan from the expected candidates per group
  const dim3 grid((unsigned)((ws.ngroups * team + 255) / 256));
  if (team == 1) hipLaunchKernelGGL(k_gather<1>, grid, dim3(256), 0, s, ws, e);
  else hipLaunchKernelGGL(k_gather<16>, grid, dim3(256), 0, s, ws, e);
}

void launch_hist(const Workspace& ws, int level, const float* e, hipStream_t s) {
  hipLaunchKernelGGL(k_hist, dim3(clamp_grid((ws.max_chunk_wgs + 1) / 2, 1024)), dim3(256), 0, s, ws, level, e);
}

void launch_select_scan(const Workspace& ws, int level, hipStream_t s) {
  hipLaunchKernelGGL(k_select_scan, dim3(ws.T), dim3(256), 0, s, ws, level);
}

void launch_count(const Workspace& ws, const float* e, hipStream_t s) {
  hipLaunchKernelGGL(k_count, dim3(clamp_grid(ws.max_chunk_wgs, 2048)), dim3(256), 0, s, ws, e);
}

void launch_chunk_scan(const Workspace& ws, hipStream_t s) {
  const int64_t blocks = ((int64_t)ws.max_chunk_wgs * 4 + kScanBlock - 1) / kScanBlock;
  hipLaunchKernelGGL(k_chunk_scan, dim3(clamp_grid(blocks, 512)), dim3(256), 0, s, ws);
}

void launch_emit(const Workspace& ws, const float* e, const OutBuf& out, hipStream_t s) {
  const dim3 grid(clamp_grid(ws.max_chunk_wgs, 2048));
  if (out.index_bits == 32)
    hipLaunchKernelGGL(k_emit<uint32_t>, grid, dim3(256), 0, s, ws, e, (uint32_t*)out.indices);
  else
    hipLaunchKernelGGL(k_emit<unsigned long long>, grid, dim3(256), 0, s, ws, e,
                       (unsigned long long*)out.indices);
}

void launch_finish(const Workspace& ws, float* e, const OutBuf& out, hipStream_t s) {
  const dim3 grid((unsigned)ws.T), blk(kFinishThreads);
  if (out.index_bits == 32)
    hipLaunchKernelGGL(k_finish<uint32_t>, grid, blk, 0, s, ws, e, (uint32_t*)out.indices, out.q, out.scales, out.block,
                       out.codec);
  else
    hipLaunchKernelGGL(k_finish<unsigned long long>, grid, blk, 0, s, ws, e, (unsigned long long*)out.indices, out.q,
                       out.scales, out.block, out.codec);
}

void launch_quant(const Workspace& ws, float* e, const OutBuf& out, int64_t ktotal, hipStream_t s) {
  if (out.codec == 1) {  // sign code: one workgroup per block
    const dim3 gridb((unsigned)ws.nblocks);
    if (out.index_bits == 32)
      hipLaunchKernelGGL(k_quant_sign<uint32_t>, gridb, dim3(256), 0, s, ws, e, (const uint32_t*)out.indices,
                         (uint8_t*)out.q, out.scales, out.block);
    else
      hipLaunchKernelGGL(k_quant_sign<unsigned long long>, gridb, dim3(256), 0, s, ws, e,
                         (const unsigned long long*)out.indices, (uint8_t*)out.q, out.scales, out.block);
    return;
  }
  const dim3 grid((unsigned)((ktotal + kQuantSpan - 1) / kQuantSpan));
  const FastDiv bdiv = make_fastdiv((uint32_t)out.block);
  if (out.index_bits == 32)
    hipLaunchKernelGGL(k_quant<uint32_t>, grid, dim3(256), 0, s, ws, e, (const uint32_t*)out.indices, out.q,
                       out.scales, out.block, bdiv, (long long)ktotal);
  else
    hipLaunchKernelGGL(k_quant<unsigned long long>, grid, dim3(256), 0, s, ws, e,
                       (const unsigned long long*)out.indices, out.q, out.scales, out.block, bdiv, (long long)ktotal);
}

}  // namespace gc
