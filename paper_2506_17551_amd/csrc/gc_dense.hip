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

// TEAM threads (64: one wavefront, blocks up to 1024; 256: the workgroup, blocks up to 8192) own
// one block. Thread `tid` of the team holds elements 4*tid .. 4*tid+3 of every row of 4*TEAM
// elements; a block is padded with zeros to P = rows * 4 * TEAM elements, rows a power of two.
template <typename G, int CODEC, int TEAM, int IB>
__global__ __launch_bounds__(256) void k_dense(const G* __restrict__ g, float* __restrict__ e, long long n,
                                               int32_t block, long long nblocks, uint8_t* __restrict__ q,
                                               float* __restrict__ scales, void* __restrict__ idx_out,
                                               uint32_t* __restrict__ flags) {
  constexpr int kTeams = 256 / TEAM;
  constexpr int kRow = TEAM * 4;
  constexpr int kMaxRows = TEAM == 256 ? 8 : 4;
  __shared__ double sh[kTeams * kRow];
  __shared__ uint32_t sh_key[4];
  const int team = threadIdx.x / TEAM, tid = threadIdx.x % TEAM, lane = threadIdx.x & 63;
  const long long b = (long long)blockIdx.x * kTeams + team;
  const bool live = b < nblocks;  // a team past the end still takes part in the barriers
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

  // ---- largest key of the block (the int8 scale; Inf/NaN detection for both codes)
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, off));
  if (TEAM == 256) {
    if (lane == 0) sh_key[threadIdx.x >> 6] = kmax;
    __syncthreads();
    kmax = max(max(sh_key[0], sh_key[1]), max(sh_key[2], sh_key[3]));
  }
  const bool finite = kmax < 0x7F800000u;

  float s;
  if (CODEC == 0) {
    s = __fdiv_rn(__uint_as_float(kmax), 127.0f);
  } else {
    // l1 norm in fp64 over the balanced tree a[i] += a[i + stride], stride = P/2 .. 1: strides of
    // a whole row or more stay inside a thread, the rest goes through LDS.
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
        for (int m = 0; m < kMaxRows / 2; ++m)
          if (m < half) {
#pragma unroll
            for (int c = 0; c < 4; ++c) r[m][c] = r[m][c] + r[m + half][c];
          }
      }
    }
    double* a = sh + team * kRow;
#pragma unroll
    for (int c = 0; c < 4; ++c) a[tid * 4 + c] = r[0][c];
    __syncthreads();
    for (int stride = kRow / 2; stride >= 1; stride >>= 1) {
      for (int i = tid; i < stride; i += TEAM) a[i] = a[i] + a[i + stride];
      __syncthreads();
    }
    s = len > 0 ? (float)(a[0] / (double)len) : 0.0f;
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
__global__ __launch_bounds__(256) void k_dense_sum(DenseDecArgs a, int W, int32_t block, long long n,
                                                   float* __restrict__ out, int weighted, float c_apply) {
  const long long i0 = ((long long)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i0 >= n) return;
  const int bytes_per_block = (block + 7) >> 3;
  float sum[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  const bool quad = (block & 3) == 0 && i0 + 4 <= n;
  if (quad) {
    const long long blk = i0 / block;
    const int r = (int)(i0 - blk * block);
#pragma unroll 4
    for (int w = 0; w < W; ++w) {
      const float s = a.scales[w][blk];
      float d[4];
      if (CODEC == 0) {
        const int8_t* qp = a.q[w] + i0;
        uint32_t word;
        if ((reinterpret_cast<uintptr_t>(qp) & 3u) == 0) {
          word = *reinterpret_cast<const uint32_t*>(qp);
        } else {
          word = (uint32_t)(uint8_t)qp[0] | ((uint32_t)(uint8_t)qp[1] << 8) | ((uint32_t)(uint8_t)qp[2] << 16) |
                 ((uint32_t)(uint8_t)qp[3] << 24);
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) d[c] = __fmul_rn((float)(int8_t)(word >> (8 * c)), s);
      } else {
        const uint32_t byte = (uint8_t)a.q[w][blk * bytes_per_block + (r >> 3)];
        const uint32_t nib = byte >> (r & 7);
#pragma unroll
        for (int c = 0; c < 4; ++c) d[c] = ((nib >> c) & 1u) ? s : -s;
      }
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (weighted) d[c] = __fdiv_rn(d[c], a.denom[w]);  // Eq. 12
        sum[c] = __fadd_rn(sum[c], d[c]);
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

template <typename G, int CODEC, int TEAM>
void launch_dense_ib(const G* g, float* e, long long n, int32_t block, long long nblocks, uint8_t* q,
                     float* scales, void* idx, int index_bits, uint32_t* flags, hipStream_t s) {
  constexpr int kTeams = 256 / TEAM;
  const dim3 grid((unsigned)((nblocks + kTeams - 1) / kTeams));
  if (!idx)
    hipLaunchKernelGGL((k_dense<G, CODEC, TEAM, 0>), grid, dim3(256), 0, s, g, e, n, block, nblocks, q, scales, idx, flags);
  else if (index_bits == 32)
    hipLaunchKernelGGL((k_dense<G, CODEC, TEAM, 32>), grid, dim3(256), 0, s, g, e, n, block, nblocks, q, scales, idx, flags);
  else
    hipLaunchKernelGGL((k_dense<G, CODEC, TEAM, 64>), grid, dim3(256), 0, s, g, e, n, block, nblocks, q, scales, idx, flags);
}

template <typename G>
void launch_dense_g(const G* g, float* e, long long n, int32_t block, long long nblocks, int codec, uint8_t* q,
                    float* scales, void* idx, int index_bits, uint32_t* flags, hipStream_t s) {
  const bool wave_team = block <= kDenseWaveBlock;
  if (codec == 0) {
    if (wave_team) launch_dense_ib<G, 0, 64>(g, e, n, block, nblocks, q, scales, idx, index_bits, flags, s);
    else launch_dense_ib<G, 0, 256>(g, e, n, block, nblocks, q, scales, idx, index_bits, flags, s);
  } else {
    if (wave_team) launch_dense_ib<G, 1, 64>(g, e, n, block, nblocks, q, scales, idx, index_bits, flags, s);
    else launch_dense_ib<G, 1, 256>(g, e, n, block, nblocks, q, scales, idx, index_bits, flags, s);
  }
}

}  // namespace

void launch_dense(const void* g, int dtype, float* e, int64_t n, int32_t block, int codec, void* q,
                  float* scales, void* idx, int index_bits, uint32_t* flags, hipStream_t s) {
  const long long nblocks = (n + block - 1) / block;
  if (dtype == 0)
    launch_dense_g<float>((const float*)g, e, n, block, nblocks, codec, (uint8_t*)q, scales, idx, index_bits, flags, s);
  else
    launch_dense_g<uint16_t>((const uint16_t*)g, e, n, block, nblocks, codec, (uint8_t*)q, scales, idx, index_bits, flags, s);
}

void launch_dense_sum(const DenseDecArgs& a, int W, int32_t block, int64_t n, int codec, float* out,
                      int weighted, int apply, float c_apply, hipStream_t s) {
  const dim3 grid((unsigned)((n + 1023) / 1024));
  if (codec == 0) {
    if (apply) hipLaunchKernelGGL((k_dense_sum<0, 1>), grid, dim3(256), 0, s, a, W, block, (long long)n, out, weighted, c_apply);
    else hipLaunchKernelGGL((k_dense_sum<0, 0>), grid, dim3(256), 0, s, a, W, block, (long long)n, out, weighted, c_apply);
  } else {
    if (apply) hipLaunchKernelGGL((k_dense_sum<1, 1>), grid, dim3(256), 0, s, a, W, block, (long long)n, out, weighted, c_apply);
    else hipLaunchKernelGGL((k_dense_sum<1, 0>), grid, dim3(256), 0, s, a, W, block, (long long)n, out, weighted, c_apply);
  }
}

}  // namespace gc
