// Dense value codes with error feedback: every entry of the accumulated gradient is sent, so
// there is no selection and no index list. With the 1-bit code this is the paper's quantizer
// (Sec. III.B, Eq. 10: signs plus one l1-based scale) applied to the whole tensor, and the
// residual of Eq. 11 carries what the signs lose into the next step.
//
//   k_dense      one pass: acc = g + e, the block statistic (amax, or the l1 norm summed in fp64
//                over the same balanced tree as the sparse path uses), the codes, and the new
//                residual acc - ghat. A block of `block` consecutive elements is owned by one
//                TEAM of threads that holds it in registers, so every element is read once.
//   k_dense_sum  the aggregate of W workers' dense codes (Eq. 8 without 1/P, optionally with the
//                damping of Eq. 12 and the update of Eq. 9), worker by worker in fp32.
// Both give, bit for bit, what the sparse path gives for k = n.
#include "gc_internal.h"

namespace gc {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned long long u64x2 __attribute__((ext_vector_type(2)));

constexpr float kMinNormal = 1.17549435e-38f;

// TEAM threads (64: one wavefront; 256: the workgroup, blocks up to 8192) own one block. Thread `tid` of the team holds elements 4*tid .. 4*tid+3 of every row of 4*TEAM
// elements; a block is padded with zeros to P = rows * 4 * TEAM elements, rows a power of two.
template <typename G, int CODEC, int TEAM, int kMaxRows>
__global__ __launch_bounds__(256) void k_dense(const G* __restrict__ g, float* __restrict__ e, long long n,
                                               int32_t block, long long nblocks, uint8_t* __restrict__ q,
                                               float* __restrict__ scales, void* __restrict__ idx_out,
                                               int IB, uint32_t* __restrict__ flags, int xcd_run) {
  constexpr int kTeams = 256 / TEAM;
  constexpr int kRow = TEAM * 4;
  __shared__ double sh[TEAM == 256 && CODEC == 1 ? 1024 : 1];
  __shared__ uint32_t sh_key[4];
  __shared__ float sh_s;
  const int team = threadIdx.x / TEAM, tid = threadIdx.x % TEAM, lane = threadIdx.x & 63;
  const long long wg = xcd_run_index(blockIdx.x, xcd_run);  // die-aware order (+3.7 % at 7B); the grid is padded
  const long long b = wg * kTeams + team;
  const bool live = b < nblocks;  // only the last workgroup can hold teams past the end (TEAM 64)
  const long long base = live ? b * (long long)block : 0;
  const int len = live ? (int)min((long long)block, n - base) : 0;
  const G* gp = g + base;
  float* ep = e + base;
  const bool vec = ((reinterpret_cast<uintptr_t>(gp) & GradVec<G>::kAlignMask) == 0) &&
                   ((reinterpret_cast<uintptr_t>(ep) & 15u) == 0);

  // ---- acc = g + e (Eq. 11), held in registers
  float acc[kMaxRows][4];
  uint32_t kmax = 0u;
#pragma unroll
  for (int m = 0; m < kMaxRows; ++m) {
    const int i0 = m * kRow + tid * 4;
    if (i0 + 4 <= len && vec) {
      const f32x4 gv = GradVec<G>::load(gp + i0);
      const f32x4 ev = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(ep + i0));
      acc[m][0] = __fadd_rn(gv.x, ev.x);
      acc[m][1] = __fadd_rn(gv.y, ev.y);
      acc[m][2] = __fadd_rn(gv.z, ev.z);
      acc[m][3] = __fadd_rn(gv.w, ev.w);
    } else {
#pragma unroll
      for (int c = 0; c < 4; ++c)
        acc[m][c] = (i0 + c < len) ? __fadd_rn(load_grad<G>(gp, i0 + c), ep[i0 + c]) : 0.0f;
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) kmax = max(kmax, key_of(acc[m][c]));
  }

  // ---- block statistics: the largest key (int8 scale; Inf/NaN detection for both codes) and, for
  // the sign code, the l1 norm in fp64 over the balanced tree a[i] += a[i + stride], stride =
  // P/2 .. 1. Element i sits in row i / kRow, thread (i % kRow) / 4, column i % 4, so strides of a
  // whole row or more are adds inside a thread, strides of 256 elements or more (TEAM 256) pair
  // wavefronts, strides 128 .. 4 pair lanes of one wavefront, strides 2 and 1 pair columns.
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, off));
  double col[4] = {0.0, 0.0, 0.0, 0.0};
  if (CODEC == 1) {
    int rows = 1;
    while (rows * kRow < len) rows <<= 1;
    double r[kMaxRows][4];
#pragma unroll
    for (int m = 0; m < kMaxRows; ++m)
#pragma unroll
      for (int c = 0; c < 4; ++c) r[m][c] = fabs((double)acc[m][c]);
#pragma unroll
    for (int half = kMaxRows / 2; half >= 1; half >>= 1) {
      if (half < rows) {
#pragma unroll
        for (int m = 0; m < (kMaxRows + 1) / 2; ++m)
          if (m < half) {
#pragma unroll
            for (int c = 0; c < 4; ++c) r[m][c] = r[m][c] + r[m + half][c];
          }
      }
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) col[c] = r[0][c];
  }
  const int wv = threadIdx.x >> 6;
  if (TEAM == 256) {
    if (CODEC == 1) {
#pragma unroll
      for (int c = 0; c < 4; ++c) sh[(wv * 4 + c) * 64 + lane] = col[c];
    }
    if (lane == 0) sh_key[wv] = kmax;
    __syncthreads();
    kmax = max(max(sh_key[0], sh_key[1]), max(sh_key[2], sh_key[3]));
    if (CODEC == 1 && wv == 0) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {  // thread offsets 128, then 64: (w0 + w2) + (w1 + w3)
        const double x1 = sh[(4 + c) * 64 + lane], x2 = sh[(8 + c) * 64 + lane], x3 = sh[(12 + c) * 64 + lane];
        col[c] = (col[c] + x2) + (x1 + x3);
      }
    }
  }
  const bool finite = kmax < 0x7F800000u;

  float s;
  if (CODEC == 0) {
    s = __fdiv_rn(__uint_as_float(kmax), 127.0f);
  } else {
    if (TEAM == 64 || wv == 0) {
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) {
#pragma unroll
        for (int c = 0; c < 4; ++c) col[c] = col[c] + __shfl_down(col[c], off);
      }
    }
    const double total = (col[0] + col[2]) + (col[1] + col[3]);  // meaningful on lane 0
    float s_lane0 = len > 0 ? (float)(total / (double)len) : 0.0f;
    if (TEAM == 256) {
      if (threadIdx.x == 0) sh_s = s_lane0;
      __syncthreads();
      s = sh_s;
    } else {
      s = __shfl(s_lane0, 0);
    }
  }
  if (!finite || !(s >= kMinNormal)) s = 0.0f;
  if (live && tid == 0) {
    scales[b] = s;
    if (!finite) flags[0] = 1u;
  }

  // ---- codes, residual, (indices)
  const int nbytes = (len + 7) >> 3;                                  // sign code: bytes of this block
  uint8_t* qb = CODEC == 0 ? q + base : q + b * (long long)((block + 7) >> 3);
#pragma unroll
  for (int m = 0; m < kMaxRows; ++m) {
    const int i0 = m * kRow + tid * 4;
    if (m * kRow >= len) break;  // uniform over the team
    float res[4];
    if (CODEC == 0) {
      uint32_t packed = 0u;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        int code = 0;
        if (s != 0.0f) {
          float rr = rintf(__fdiv_rn(acc[m][c], s));
          rr = fminf(fmaxf(rr, -127.0f), 127.0f);
          code = (int)rr;
        }
        res[c] = __fsub_rn(acc[m][c], __fmul_rn((float)code, s));
        packed |= ((uint32_t)code & 0xFFu) << (8 * c);
      }
      if (i0 + 4 <= len && (reinterpret_cast<uintptr_t>(qb + i0) & 3u) == 0) {
        *reinterpret_cast<uint32_t*>(qb + i0) = packed;
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (i0 + c < len) qb[i0 + c] = (uint8_t)(packed >> (8 * c));
      }
    } else {
      uint32_t nib = 0u;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bool plus = acc[m][c] >= 0.0f;
        res[c] = __fsub_rn(acc[m][c], plus ? s : -s);
        if (plus && finite && i0 + c < len) nib |= 1u << c;
      }
      // 8 neighbouring lanes hold the 32 sign bits of 32 consecutive elements
      uint32_t x = nib | ((uint32_t)__shfl_down((int)nib, 1) << 4);   // a byte, on even lanes
      const uint32_t y = x | ((uint32_t)__shfl_down((int)x, 2) << 8);
      const uint32_t z = y | ((uint32_t)__shfl_down((int)y, 4) << 16);  // a word, on every 8th lane
      const int lead = i0 - (lane & 7) * 4;                             // first element of the word
      const bool word_ok = (lead >> 3) + 4 <= nbytes && (reinterpret_cast<uintptr_t>(qb + (lead >> 3)) & 3u) == 0;
      if (word_ok) {
        if ((lane & 7) == 0) *reinterpret_cast<uint32_t*>(qb + (i0 >> 3)) = z;
      } else if ((lane & 1) == 0 && i0 < len) {
        qb[i0 >> 3] = (uint8_t)x;
      }
    }
    if (i0 + 4 <= len && vec) {
      const f32x4 rv = {res[0], res[1], res[2], res[3]};
      __builtin_nontemporal_store(rv, reinterpret_cast<f32x4*>(ep + i0));
    } else {
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (i0 + c < len) ep[i0 + c] = res[c];
    }
    if (IB == 32) {
      uint32_t* ip = static_cast<uint32_t*>(idx_out) + base + i0;
      const uint32_t v0 = (uint32_t)(base + i0);
      if (i0 + 4 <= len && (reinterpret_cast<uintptr_t>(ip) & 15u) == 0) {
        const u32x4 iv = {v0, v0 + 1u, v0 + 2u, v0 + 3u};
        *reinterpret_cast<u32x4*>(ip) = iv;
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (i0 + c < len) ip[c] = v0 + (uint32_t)c;
      }
    } else if (IB == 64) {
      unsigned long long* ip = static_cast<unsigned long long*>(idx_out) + base + i0;
      const unsigned long long v0 = (unsigned long long)(base + i0);
      if (i0 + 4 <= len && (reinterpret_cast<uintptr_t>(ip) & 15u) == 0) {
        const u64x2 lo = {v0, v0 + 1ull}, hi = {v0 + 2ull, v0 + 3ull};
        *reinterpret_cast<u64x2*>(ip) = lo;
        *reinterpret_cast<u64x2*>(ip + 2) = hi;
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (i0 + c < len) ip[c] = v0 + (unsigned long long)c;
      }
    }
  }
}

// Aggregate of W workers' dense codes. A thread owns 4 consecutive elements; when block is a
// multiple of 4 they share a block (one scale, one code word or one nibble per worker).
// MODE 0: out = sum. MODE 1: theta -= fl32(step * sum) (Eq. 9).
template <int CODEC, int MODE>
__device__ __forceinline__ void dense_sum_quad(const DenseDecArgs& a, int W, int32_t block, long long i0,
                                               long long n, float* __restrict__ out, int weighted,
                                               float c_apply) {
  if (i0 >= n) return;
  const int bytes_per_block = (block + 7) >> 3;
  float sum[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  const bool quad = (block & 3) == 0 && i0 + 4 <= n;
  if (quad) {
    const long long blk = i0 / block;
    const int r = (int)(i0 - blk * block);
    const long long qoff = CODEC == 0 ? i0 : blk * bytes_per_block + (r >> 3);
    const int shift = r & 7;  // sign code: 0 or 4, the thread's nibble inside its byte
    constexpr int kBatch = 16;  // loads of this many workers are in flight together
    for (int w0 = 0; w0 < W; w0 += kBatch) {
      uint32_t code[kBatch];
      float sc[kBatch];
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        if (w0 + j < W) {
          sc[j] = a.scales[w0 + j][blk];
          const int8_t* qp = a.q[w0 + j] + qoff;
          if (CODEC == 1) {
            code[j] = (uint8_t)qp[0];
          } else if ((reinterpret_cast<uintptr_t>(qp) & 3u) == 0) {
            code[j] = *reinterpret_cast<const uint32_t*>(qp);
          } else {
            code[j] = (uint32_t)(uint8_t)qp[0] | ((uint32_t)(uint8_t)qp[1] << 8) |
                      ((uint32_t)(uint8_t)qp[2] << 16) | ((uint32_t)(uint8_t)qp[3] << 24);
          }
        }
      }
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        if (w0 + j < W) {
          const float s = sc[j];
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            float d;
            if (CODEC == 0) d = __fmul_rn((float)(int8_t)(code[j] >> (8 * c)), s);
            else d = ((code[j] >> (shift + c)) & 1u) ? s : -s;
            if (weighted) d = __fdiv_rn(d, a.denom[w0 + j]);  // Eq. 12
            sum[c] = __fadd_rn(sum[c], d);
          }
        }
      }
    }
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const long long i = i0 + c;
      if (i >= n) break;
      const long long blk = i / block;
      const int r = (int)(i - blk * block);
      for (int w = 0; w < W; ++w) {
        const float s = a.scales[w][blk];
        float d;
        if (CODEC == 0) {
          d = __fmul_rn((float)a.q[w][i], s);
        } else {
          const uint32_t byte = (uint8_t)a.q[w][blk * bytes_per_block + (r >> 3)];
          d = ((byte >> (r & 7)) & 1u) ? s : -s;
        }
        if (weighted) d = __fdiv_rn(d, a.denom[w]);
        sum[c] = __fadd_rn(sum[c], d);
      }
    }
  }
  float* op = out + i0;
  if (i0 + 4 <= n && (reinterpret_cast<uintptr_t>(op) & 15u) == 0) {
    if (MODE == 0) {
      const f32x4 v = {sum[0], sum[1], sum[2], sum[3]};
      __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(op));
    } else {
      f32x4 th = *reinterpret_cast<const f32x4*>(op);
      th.x = __fsub_rn(th.x, __fmul_rn(c_apply, sum[0]));
      th.y = __fsub_rn(th.y, __fmul_rn(c_apply, sum[1]));
      th.z = __fsub_rn(th.z, __fmul_rn(c_apply, sum[2]));
      th.w = __fsub_rn(th.w, __fmul_rn(c_apply, sum[3]));
      *reinterpret_cast<f32x4*>(op) = th;
    }
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if (i0 + c >= n) break;
      if (MODE == 0) op[c] = sum[c];
      else op[c] = __fsub_rn(op[c], __fmul_rn(c_apply, sum[c]));
    }
  }
}

// A workgroup covers kDenseSumIter * 1024 consecutive elements, 1024 at a time: larger contiguous
// pieces per workgroup raise the store rate of this write-dominated kernel.
constexpr int kDenseSumIter = 4;
template <int CODEC, int MODE>
__global__ __launch_bounds__(256) void k_dense_sum(DenseDecArgs a, int W, int32_t block, long long start,
                                                   long long n, float* __restrict__ out, int weighted,
                                                   float c_apply) {
#pragma unroll 1
  for (int it = 0; it < kDenseSumIter; ++it) {
    const long long i0 = start + (((long long)blockIdx.x * kDenseSumIter + it) * 256 + threadIdx.x) * 4;
    dense_sum_quad<CODEC, MODE>(a, W, block, i0, n, out, weighted, c_apply);
  }
}

// Aggregate of W workers' sign codes when block is a multiple of 512 (the bit stream then has no
// padding but at the very end, and a tile has one scale per worker). A wavefront owns a tile of 512
// elements, lane l the elements 64 j + l, j = 0..7: the 64 sign bits of row j of a worker are one
// 64-bit word that is the same for the whole wavefront, so it is fetched through the scalar path
// and used directly as the lane mask of the select between +s and -s: two vector instructions per
// element and worker (select, add), in worker order. Lane w keeps worker w's scale (already
// divided by 1 + staleness, Eq. 12). The scalar fetches of one wavefront are serial, so the tile's
// words of every worker are first touched with one wide vector load, which brings them into L2.
constexpr int kSignTileRows = 8;
constexpr int kSignTile = 64 * kSignTileRows;
constexpr int kSignBatch = 4;  // workers whose words are fetched together

template <int NW>
__device__ __forceinline__ void sign_tile_workers(const DenseDecArgs& a, int w0, long long tile, float sv,
                                                  float (&sum)[kSignTileRows]) {
  unsigned long long m[NW][kSignTileRows];
  float d[NW];
#pragma unroll
  for (int u = 0; u < NW; ++u) d[u] = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(sv), w0 + u));
#pragma unroll
  for (int u = 0; u < NW; ++u) {
    const unsigned long long* __restrict__ qw =
        reinterpret_cast<const unsigned long long*>(a.q[w0 + u]) + tile * kSignTileRows;
#pragma unroll
    for (int j = 0; j < kSignTileRows; ++j) m[u][j] = qw[j];
  }
#pragma unroll
  for (int u = 0; u < NW; ++u) {  // worker order
#pragma unroll
    for (int j = 0; j < kSignTileRows; ++j) {
      const bool plus = __builtin_amdgcn_inverse_ballot_w64(m[u][j]);
      sum[j] = __fadd_rn(sum[j], plus ? d[u] : -d[u]);
    }
  }
}

template <int MODE>
__global__ __launch_bounds__(256) void k_dense_sum_sign(DenseDecArgs a, int W, int32_t block, long long ntiles,
                                                        float* __restrict__ out, int weighted, float c_apply) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  // plain order: for this write-dominated kernel runs per compute die measured 8 % slower
  const long long tile = (long long)blockIdx.x * 4 + wave;
  if (tile >= ntiles) return;
  const long long ebase = tile * kSignTile;
  // touch the tile's 64 bytes of every worker: 4 lanes per worker, 16 workers per load
  u32x4 touch[kMaxWorkers / 16];
#pragma unroll
  for (int r = 0; r < kMaxWorkers / 16; ++r) {
    const int w = r * 16 + (lane >> 2);
    touch[r] = u32x4{0u, 0u, 0u, 0u};
    if (w < W) touch[r] = *reinterpret_cast<const u32x4*>(a.q[w] + tile * (kSignTile / 8) + (lane & 3) * 16);
  }
  float sv = 0.0f;
  if (lane < W) {
    sv = a.scales[lane][ebase / block];
    if (weighted) sv = __fdiv_rn(sv, a.denom[lane]);  // (-s) / denom == -(s / denom)
  }
  float sum[kSignTileRows];
#pragma unroll
  for (int j = 0; j < kSignTileRows; ++j) sum[j] = 0.0f;
  int w = 0;
  for (; w + kSignBatch <= W; w += kSignBatch) sign_tile_workers<kSignBatch>(a, w, tile, sv, sum);
  for (; w < W; ++w) sign_tile_workers<1>(a, w, tile, sv, sum);
  float* op = out + ebase + lane;
#pragma unroll
  for (int j = 0; j < kSignTileRows; ++j) {
    if (MODE == 0) __builtin_nontemporal_store(sum[j], op + 64 * j);
    else op[64 * j] = __fsub_rn(op[64 * j], __fmul_rn(c_apply, sum[j]));
  }
#pragma unroll
  for (int r = 0; r < kMaxWorkers / 16; ++r)  // keeps the touching loads alive without using them
    asm volatile("" ::"v"(touch[r].x), "v"(touch[r].y), "v"(touch[r].z), "v"(touch[r].w));
}

template <typename G, int CODEC, int TEAM, int ROWS>
void launch_dense_k(const G* g, float* e, long long n, int32_t block, long long nblocks, uint8_t* q,
                    float* scales, void* idx, int index_bits, uint32_t* flags, int lds_pad, hipStream_t s) {
  constexpr int kTeams = 256 / TEAM;
  const int64_t wgs = (nblocks + kTeams - 1) / kTeams;
  const int run = xcd_run_for((int64_t)kTeams * block);
  const dim3 grid((unsigned)xcd_run_grid(wgs, run));
  hipLaunchKernelGGL((k_dense<G, CODEC, TEAM, ROWS>), grid, dim3(256), (size_t)lds_pad, s, g, e, n, block, nblocks, q,
                     scales, idx, idx ? index_bits : 0, flags, run);
}

// A block is held by one wavefront (up to `wave_block` elements, at most 2048) or by the workgroup;
// the row count is the smallest power of two that covers the block.
template <typename G, int CODEC>
void launch_dense_c(const G* g, float* e, long long n, int32_t block, long long nblocks, uint8_t* q,
                    float* scales, void* idx, int index_bits, uint32_t* flags, int wave_block, int lds_pad,
                    hipStream_t s) {
#define GC_DENSE(TEAM, ROWS) \
  launch_dense_k<G, CODEC, TEAM, ROWS>(g, e, n, block, nblocks, q, scales, idx, index_bits, flags, lds_pad, s)
  const bool wave_team = block <= wave_block && block <= 2048;
  // Workgroup teams of 2048 elements and more measured fastest on the 7B workload with 5-6 workgroups
  // per compute unit (the sign coder holds 8 KB of LDS of its own); elsewhere occupancy matters little.
  if (lds_pad < 0) lds_pad = wave_team ? 0 : (CODEC == 1 ? 16384 : 32768);
  if (wave_team) {
    if (block <= 256) GC_DENSE(64, 1);
    else if (block <= 512) GC_DENSE(64, 2);
    else if (block <= 1024) GC_DENSE(64, 4);
    else GC_DENSE(64, 8);
  } else {
    if (block <= 1024) GC_DENSE(256, 1);
    else if (block <= 2048) GC_DENSE(256, 2);
    else if (block <= 4096) GC_DENSE(256, 4);
    else GC_DENSE(256, 8);
  }
#undef GC_DENSE
}

template <typename G>
void launch_dense_g(const G* g, float* e, long long n, int32_t block, long long nblocks, int codec, uint8_t* q,
                    float* scales, void* idx, int index_bits, uint32_t* flags, int wave_block, int lds_pad,
                    hipStream_t s) {
  if (codec == 0) launch_dense_c<G, 0>(g, e, n, block, nblocks, q, scales, idx, index_bits, flags, wave_block, lds_pad, s);
  else launch_dense_c<G, 1>(g, e, n, block, nblocks, q, scales, idx, index_bits, flags, wave_block, lds_pad, s);
}

}  // namespace

void launch_dense(const void* g, int dtype, float* e, int64_t n, int32_t block, int codec, void* q,
                  float* scales, void* idx, int index_bits, uint32_t* flags, int wave_block, int lds_pad,
                  hipStream_t s) {
  const long long nblocks = (n + block - 1) / block;
  if (dtype == 0)
    launch_dense_g<float>((const float*)g, e, n, block, nblocks, codec, (uint8_t*)q, scales, idx, index_bits, flags,
                          wave_block, lds_pad, s);
  else
    launch_dense_g<uint16_t>((const uint16_t*)g, e, n, block, nblocks, codec, (uint8_t*)q, scales, idx, index_bits,
                             flags, wave_block, lds_pad, s);
}

void launch_dense_sum(const DenseDecArgs& a, int W, int32_t block, int64_t n, int codec, float* out,
                      int weighted, int apply, float c_apply, hipStream_t s) {
  long long start = 0;
  if (codec == 1 && block % kSignTile == 0) {
    bool aligned = true;
    for (int w = 0; w < W; ++w) aligned = aligned && (reinterpret_cast<uintptr_t>(a.q[w]) % 16 == 0);
    const long long ntiles = n / kSignTile;  // whole tiles; the rest goes through the generic kernel
    if (aligned && ntiles > 0) {
      const dim3 grid((unsigned)((ntiles + 3) / 4));
      if (apply) hipLaunchKernelGGL((k_dense_sum_sign<1>), grid, dim3(256), 0, s, a, W, block, ntiles, out, weighted, c_apply);
      else hipLaunchKernelGGL((k_dense_sum_sign<0>), grid, dim3(256), 0, s, a, W, block, ntiles, out, weighted, c_apply);
      start = ntiles * kSignTile;
      if (start >= n) return;
    }
  }
  const dim3 grid((unsigned)((n - start + 1024 * kDenseSumIter - 1) / (1024 * kDenseSumIter)));
#define GC_DSUM(C, M) \
  hipLaunchKernelGGL((k_dense_sum<C, M>), grid, dim3(256), 0, s, a, W, block, start, (long long)n, out, weighted, c_apply)
  if (codec == 0) {
    if (apply) GC_DSUM(0, 1); else GC_DSUM(0, 0);
  } else {
    if (apply) GC_DSUM(1, 1); else GC_DSUM(1, 0);
  }
#undef GC_DSUM
}

}  // namespace gc
