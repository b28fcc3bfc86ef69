// Row-sparse gradients: the gradient of an embedding table arrives as U touched rows (ascending,
// unique row ids) and their U x D values, while the error-feedback residual of Eq. 11 lives with
// the table (R x D). The step runs on the touched rows only: their residual rows are gathered into
// a compact U x D tensor, the flat compress path runs on it, and afterwards the new residual rows
// are scattered back and the compact positions are rewritten as positions in the table. Rows are
// contiguous runs of D floats, so both copies are coalesced.
#include "gc_internal.h"

namespace gc {
namespace {

// A row id must lie in [0, R) and exceed its predecessor. A bad id is never dereferenced: its
// values are gathered as zeros, nothing is scattered for it, and the call is flagged.
__device__ __forceinline__ bool row_ok(const long long* __restrict__ rows, long long u, long long R) {
  const long long r = rows[u];
  return r >= 0 && r < R && (u == 0 || rows[u - 1] < r);
}

// VEC = 4: D is a multiple of 4 and both arrays are 16-byte aligned; VEC = 1 otherwise.
template <int VEC>
__global__ __launch_bounds__(256) void k_rows_gather(const float* __restrict__ table,
                                                     const long long* __restrict__ rows, long long U,
                                                     long long D, long long R, float* __restrict__ ec,
                                                     uint32_t* __restrict__ flags) {
  const long long t = ((long long)blockIdx.x * 256 + threadIdx.x) * VEC;
  if (t >= U * D) return;
  const long long u = t / D, c = t - u * D;
  const bool ok = row_ok(rows, u, R);
  if (!ok && c == 0) flags[1] = 1u;
  if (VEC == 4) {
    f32x4 v = {0.0f, 0.0f, 0.0f, 0.0f};
    if (ok) v = *reinterpret_cast<const f32x4*>(table + rows[u] * D + c);
    *reinterpret_cast<f32x4*>(ec + t) = v;
  } else {
    ec[t] = ok ? table[rows[u] * D + c] : 0.0f;
  }
}

// Scatter the new residual rows back, and rewrite the k compact positions as table positions.
template <int VEC, typename I>
__global__ __launch_bounds__(256) void k_rows_finish(float* __restrict__ table, const long long* __restrict__ rows,
                                                     long long U, long long D, long long R,
                                                     const float* __restrict__ ec,
                                                     const uint32_t* __restrict__ compact_idx, long long k,
                                                     I* __restrict__ out_idx) {
  const long long tid = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long t = tid * VEC;
  if (t < U * D) {
    const long long u = t / D, c = t - u * D;
    if (row_ok(rows, u, R)) {
      if (VEC == 4) *reinterpret_cast<f32x4*>(table + rows[u] * D + c) = *reinterpret_cast<const f32x4*>(ec + t);
      else table[rows[u] * D + c] = ec[t];
    }
  }
  if (tid < k) {
    const long long p = (long long)compact_idx[tid];
    const long long u = p / D, c = p - u * D;
    out_idx[tid] = row_ok(rows, u, R) ? (I)(rows[u] * D + c) : (I)0;
  }
}

// Table positions (row * D + column) of one worker's pairs rewritten as positions in the compact
// (Ru x D) output over the row list urows. lower_bound is monotone, so the rewritten positions stay
// ascending; a row that is missing from the list is flagged and lands on a neighbouring listed row
// (the result is then unspecified, but every position stays inside the output).
// All workers in one launch: blockIdx.y is the worker, whose compact positions go to out + at[w].
__global__ __launch_bounds__(256) void k_rows_remap(RowsRemapArgs a, const long long* __restrict__ urows, long long Ru,
                                                    long long D, uint32_t* __restrict__ out,
                                                    uint32_t* __restrict__ flags) {
  const int w = blockIdx.y;
  const long long j = (long long)blockIdx.x * 256 + threadIdx.x;
  if (j >= (long long)a.k[w]) return;
  const unsigned long long pos = a.bits[w] == 32 ? (unsigned long long)static_cast<const uint32_t*>(a.idx[w])[j]
                                                 : static_cast<const unsigned long long*>(a.idx[w])[j];
  const long long row = (long long)(pos / (unsigned long long)D);
  const long long col = (long long)(pos - (unsigned long long)row * (unsigned long long)D);
  long long lo = 0, hi = Ru;  // first r with urows[r] >= row
  while (lo < hi) {
    const long long mid = lo + ((hi - lo) >> 1);
    if (urows[mid] < row) lo = mid + 1; else hi = mid;
  }
  if (lo >= Ru || urows[lo] != row) {
    flags[1] = 1u;
    if (lo >= Ru) lo = Ru - 1;
  }
  out[a.at[w] + j] = (uint32_t)(lo * D + col);
}

}  // namespace

void launch_rows_remap(const RowsRemapArgs& a, int W, const long long* urows, int64_t Ru, int64_t D, uint32_t* out,
                       uint32_t* flags, hipStream_t s) {
  uint32_t kmax = 0;
  for (int w = 0; w < W; ++w) kmax = a.k[w] > kmax ? a.k[w] : kmax;
  if (kmax == 0) return;
  const dim3 grid((unsigned)((kmax + 255) / 256), (unsigned)W);
  hipLaunchKernelGGL(k_rows_remap, grid, dim3(256), 0, s, a, urows, (long long)Ru, (long long)D, out, flags);
}

void launch_rows_gather(const float* table, const long long* rows, int64_t U, int64_t D, int64_t R, float* ec,
                        uint32_t* flags, hipStream_t s) {
  const bool vec = D % 4 == 0 && reinterpret_cast<uintptr_t>(table) % 16 == 0 && reinterpret_cast<uintptr_t>(ec) % 16 == 0;
  const int64_t threads = vec ? U * D / 4 : U * D;
  const dim3 grid((unsigned)((threads + 255) / 256));
  if (vec) hipLaunchKernelGGL(k_rows_gather<4>, grid, dim3(256), 0, s, table, rows, (long long)U, (long long)D, (long long)R, ec, flags);
  else hipLaunchKernelGGL(k_rows_gather<1>, grid, dim3(256), 0, s, table, rows, (long long)U, (long long)D, (long long)R, ec, flags);
}

void launch_rows_finish(float* table, const long long* rows, int64_t U, int64_t D, int64_t R, const float* ec,
                        const uint32_t* compact_idx, int64_t k, void* out_idx, int index_bits, hipStream_t s) {
  const bool vec = D % 4 == 0 && reinterpret_cast<uintptr_t>(table) % 16 == 0 && reinterpret_cast<uintptr_t>(ec) % 16 == 0;
  const int64_t copy_threads = vec ? U * D / 4 : U * D;
  const int64_t threads = copy_threads > k ? copy_threads : k;
  const dim3 grid((unsigned)((threads + 255) / 256));
#define GC_ROWS_FINISH(VEC, ITYPE)                                                                           \
  hipLaunchKernelGGL((k_rows_finish<VEC, ITYPE>), grid, dim3(256), 0, s, table, rows, (long long)U, (long long)D, \
                     (long long)R, ec, compact_idx, (long long)k, (ITYPE*)out_idx)
  if (index_bits == 32) {
    if (vec) GC_ROWS_FINISH(4, uint32_t); else GC_ROWS_FINISH(1, uint32_t);
  } else {
    if (vec) GC_ROWS_FINISH(4, unsigned long long); else GC_ROWS_FINISH(1, unsigned long long);
  }
#undef GC_ROWS_FINISH
}

}  // namespace gc
