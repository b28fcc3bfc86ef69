// CPU oracle for error-feedback top-k gradient compression with per-block int8
// quantization, and for the decompress-and-sum aggregate.
//
// THIS FILE IS TEST INFRASTRUCTURE. It is the slow, single-threaded, obviously
// correct statement of what the method computes. Nothing in the product path
// (the HIP library, its Python binding) may include, link or call it; only the
// tests, the smoke check and the benchmark's cpu_baseline leg do. It shares no
// code, header, table or constant with the HIP path.
//
// What the paper fixes (Sec. III.B):
//   * Top-k sparsification sends the k entries of largest magnitude and keeps
//     the rest as a residual; Eq. (11): r_{t+1} = r_t + g - ghat.
//   * The aggregate of the workers' gradients is their mean, Eq. (8); this file
//     returns the plain sum (the 1/P factor is the caller's scalar).
// What the paper leaves open and this oracle fixes (each is a stated reading):
//   R1  The selection runs on acc = r_t + g (one fp32 add), not on g alone, and
//       r_{t+1} = acc - ghat.
//   R2  "Largest absolute" compares the 31 magnitude bits of the fp32 pattern as
//       an unsigned integer; +0 and -0 tie; subnormals keep their order.
//   R3  Ties at the k-th magnitude go to the lower index, so the kept set is
//       unique. Kept indices are reported in ascending order.
//   R4  The 8-bit code is symmetric abs-max int8 over blocks of `block`
//       consecutive KEPT entries (in ascending-index order; last block may be
//       short): s = amax / 127 (IEEE divide), q = clamp(rint(v / s), -127, 127)
//       with round-half-to-even; a block whose scale is zero or subnormal gets
//       s = 0 and all codes 0.
//   R5  ghat at a kept position is fl32(q * s); the residual there is
//       fl32(acc - fl32(q*s)) (two roundings, never fused). Elsewhere ghat = 0
//       and the residual is acc itself.
//   R6  k = clamp(ceil(n * density), 1, n) evaluated in IEEE double.
//   R7  Non-finite acc inside a kept block is reported as an error.
//   R8  The sum over workers is accumulated in fp32 in ascending worker order,
//       starting from +0.
//   R9  Alternative value code, the paper's own 1-bit quantizer (Eq. 10): the code of a kept
//       entry is its sign (+1 if v >= 0, which includes -0; -1 otherwise) and the block's
//       scale is the mean magnitude ||v||_1 / len (Sec. III.B, Eq. 10: the scale is derived
//       from the l1 norm). To make the scale a fixed number, the l1 sum is accumulated in fp64
//       by the balanced binary tree over the block's entries padded with zeros to a power of
//       two, s = (float)(sum / len) (one fp64 division, one rounding to fp32), zero or
//       subnormal s sends zeros. The tree is a CHOSEN order, not a plain definition: it is the
//       order a parallel reduction can reproduce bit for bit. The pins therefore also check the
//       sent scale against the plain left-to-right fp64 sum and the exactly rounded sum. ghat = +-s; the residual is fl32(acc - ghat). Signs are
//       packed 8 per byte, least significant bit first, every block starting a new byte.
//   R10 Row-sparse gradients (an embedding table of R rows x D columns of which a step touches
//       U rows): the residual lives with the table, the step runs on the touched rows only -
//       acc = vals + residual[rows], top-k over those U*D entries, residual[rows] rewritten -
//       so untouched rows neither compete nor change, and indices are reported as positions in
//       the table, row * D + column (ascending, since the rows are given ascending).
// Parity status: the selection (R1-R3), Eq. (11) and Eq. (8) are pinned by the
// CPU tests (brute-force sort, exact invariants, closed-form quantiles). The
// choice of int8 scheme (R4), block semantics and the k rounding rule (R6) are
// "parity unpinned" by the paper: it prints no scheme and no worked example;
// they are pinned only to the hand-worked cases under tests/golden/.
//
// Build: g++ -O2 -std=c++17 -ffp-contract=off -fno-fast-math -shared -fPIC

#include <algorithm>
#include <cfloat>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <functional>
#include <vector>

namespace {

inline float widen(const void* g, int dtype, int64_t i) {
  if (dtype == 0) return static_cast<const float*>(g)[i];
  // bfloat16: the upper 16 bits of a binary32 pattern; widening is exact.
  uint32_t bits = static_cast<uint32_t>(static_cast<const uint16_t*>(g)[i]) << 16;
  float f;
  std::memcpy(&f, &bits, 4);
  return f;
}

inline uint32_t magnitude_key(float x) {
  uint32_t b;
  std::memcpy(&b, &x, 4);
  return b & 0x7FFFFFFFu;
}

}  // namespace

extern "C" {

enum { GCO_OK = 0, GCO_ERR_INVALID_ARG = 1, GCO_ERR_NONFINITE = 4 };

// Reading R6.
int64_t gco_k_from_density(int64_t n, double density) {
  if (n <= 0) return 0;
  double kd = std::ceil(static_cast<double>(n) * density);
  if (!(kd >= 1.0)) return 1;
  if (kd >= static_cast<double>(n)) return n;
  return static_cast<int64_t>(kd);
}

// Bytes of code for k kept entries: one per entry (int8), or the packed sign bits of each
// block rounded up to whole bytes (sign code).
int64_t gco_num_code_bytes(int64_t k, int32_t block, int32_t codec) {
  if (k <= 0 || block < 1) return 0;
  if (codec == 0) return k;
  const int64_t full = k / block, rest = k % block;
  return full * ((block + 7) / 8) + (rest + 7) / 8;
}

// One worker, one tensor, one error-feedback step (Sec. III.B, Eq. 11).
//   g        n gradient entries, dtype 0 = fp32, 1 = bf16            (read only)
//   e        n fp32 residual entries: r_t on entry, r_{t+1} on return
//   idx      k kept indices, ascending; uint32 if index_bits == 32 else uint64
//   q        k int8 codes, same order
//   scales   ceil(k / block) fp32 scales
//   codec    0: per-block int8 (R4), 1: per-block sign bit with mean-magnitude scale (R9)
int gco_compress_codec(const void* g, int dtype, float* e, int64_t n, int64_t k, int32_t block,
                       void* idx, int32_t index_bits, int8_t* q, float* scales, int32_t codec) {
  if (!g || !e || !idx || !q || !scales) return GCO_ERR_INVALID_ARG;
  if (codec != 0 && codec != 1) return GCO_ERR_INVALID_ARG;
  if (n <= 0 || k < 1 || k > n || block < 1) return GCO_ERR_INVALID_ARG;
  if (dtype != 0 && dtype != 1) return GCO_ERR_INVALID_ARG;
  if (index_bits != 32 && index_bits != 64) return GCO_ERR_INVALID_ARG;
  if (index_bits == 32 && n > (int64_t(1) << 32)) return GCO_ERR_INVALID_ARG;

  // acc = g + r_t, one binary32 addition per entry (R1).
  std::vector<float> acc(n);
  for (int64_t i = 0; i < n; ++i) acc[i] = widen(g, dtype, i) + e[i];

  // Magnitude keys (R2) and the k-th largest of them.
  std::vector<uint32_t> key(n);
  for (int64_t i = 0; i < n; ++i) key[i] = magnitude_key(acc[i]);
  uint32_t T;
  {
    std::vector<uint32_t> work(key);
    std::nth_element(work.begin(), work.begin() + (k - 1), work.end(), std::greater<uint32_t>());
    T = work[k - 1];
  }
  int64_t c_gt = 0;
  for (int64_t i = 0; i < n; ++i) c_gt += (key[i] > T);
  const int64_t quota = k - c_gt;  // how many entries equal to T are kept (R3)

  // Kept set in ascending index order; ties at T go to the lowest indices.
  std::vector<int64_t> kept(k);
  std::vector<float> v(k);
  {
    int64_t j = 0, taken = 0;
    for (int64_t i = 0; i < n; ++i) {
      bool keep = key[i] > T;
      if (!keep && key[i] == T && taken < quota) {
        keep = true;
        ++taken;
      }
      if (keep) {
        if (j >= k) return GCO_ERR_INVALID_ARG;  // cannot happen
        kept[j] = i;
        v[j] = acc[i];
        ++j;
      }
    }
    if (j != k) return GCO_ERR_INVALID_ARG;  // cannot happen
  }

  // Entries that are not kept: the residual is acc (Eq. 11 with ghat = 0).
  for (int64_t i = 0; i < n; ++i) e[i] = acc[i];

  // Per-block int8 codes (R4) and the residual at kept entries (R5).
  int status = GCO_OK;
  const int64_t nblocks = (k + block - 1) / block;
  for (int64_t b = 0; b < nblocks; ++b) {
    const int64_t j0 = b * block;
    const int64_t j1 = std::min<int64_t>(k, j0 + block);
    float amax = 0.0f;
    bool finite = true;
    for (int64_t j = j0; j < j1; ++j) {
      if (!std::isfinite(v[j])) finite = false;
      float a = std::fabs(v[j]);
      if (a > amax) amax = a;
    }
    if (codec == 1) {  // Eq. 10: sign bits and one scale per block
      const int64_t len = j1 - j0;
      uint8_t* bytes = reinterpret_cast<uint8_t*>(q) + b * ((block + 7) / 8);
      for (int64_t r = 0; r < (len + 7) / 8; ++r) bytes[r] = 0;
      if (!finite) {
        status = GCO_ERR_NONFINITE;
        scales[b] = 0.0f;
        continue;
      }
      int64_t P = 1;
      while (P < len) P <<= 1;
      std::vector<double> tree(P, 0.0);
      for (int64_t r = 0; r < len; ++r) tree[r] = std::fabs(static_cast<double>(v[j0 + r]));
      for (int64_t stride = P / 2; stride >= 1; stride /= 2)
        for (int64_t r = 0; r < stride; ++r) tree[r] = tree[r] + tree[r + stride];
      float s1 = static_cast<float>(tree[0] / static_cast<double>(len));
      if (!(s1 >= FLT_MIN)) s1 = 0.0f;
      scales[b] = s1;
      for (int64_t r = 0; r < len; ++r) {
        const float val = v[j0 + r];
        const bool plus = val >= 0.0f;
        if (plus) bytes[r / 8] = static_cast<uint8_t>(bytes[r / 8] | (1u << (r % 8)));
        const float d = plus ? s1 : -s1;
        e[kept[j0 + r]] = val - d;
      }
      continue;
    }
    if (!finite) {
      status = GCO_ERR_NONFINITE;
      scales[b] = 0.0f;
      for (int64_t j = j0; j < j1; ++j) q[j] = 0;
      continue;
    }
    float s = amax / 127.0f;
    if (!(s >= FLT_MIN)) s = 0.0f;
    scales[b] = s;
    for (int64_t j = j0; j < j1; ++j) {
      int code = 0;
      if (s != 0.0f) {
        float t = std::nearbyintf(v[j] / s);  // default rounding mode: to nearest even
        if (t > 127.0f) t = 127.0f;
        if (t < -127.0f) t = -127.0f;
        code = static_cast<int>(t);
      }
      q[j] = static_cast<int8_t>(code);
      volatile float d = static_cast<float>(code) * s;  // rounded to fp32 on its own
      e[kept[j]] = v[j] - d;
    }
  }

  if (index_bits == 32) {
    uint32_t* o = static_cast<uint32_t*>(idx);
    for (int64_t j = 0; j < k; ++j) o[j] = static_cast<uint32_t>(kept[j]);
  } else {
    uint64_t* o = static_cast<uint64_t*>(idx);
    for (int64_t j = 0; j < k; ++j) o[j] = static_cast<uint64_t>(kept[j]);
  }
  return status;
}

int gco_compress(const void* g, int dtype, float* e, int64_t n, int64_t k, int32_t block,
                 void* idx, int32_t index_bits, int8_t* q, float* scales) {
  return gco_compress_codec(g, dtype, e, n, k, block, idx, index_bits, q, scales, 0);
}

// A list of tensors laid out back to back in one flat buffer; each tensor gets
// its own top-k and its own quantization blocks (blocks never straddle
// tensors). Outputs are concatenated in tensor order; indices are positions in
// the FLAT buffer, so the concatenation is again ascending.
//   offsets  T+1 element offsets, offsets[0] = 0, non-decreasing
//   k        T per-tensor counts (k[t] in [1, n_t])
//   scales   sum_t ceil(k[t]/block) entries
int gco_compress_multi_codec(const void* g, int dtype, float* e, const int64_t* offsets,
                             const int64_t* k, int32_t T, int32_t block, void* idx,
                             int32_t index_bits, int8_t* q, float* scales, int32_t codec) {
  if (!offsets || !k || T < 1) return GCO_ERR_INVALID_ARG;
  int status = GCO_OK;
  int64_t kpos = 0, spos = 0, qpos = 0;
  for (int32_t t = 0; t < T; ++t) {
    const int64_t off = offsets[t];
    const int64_t n = offsets[t + 1] - off;
    if (n <= 0) return GCO_ERR_INVALID_ARG;
    const void* gt = (dtype == 0)
                         ? static_cast<const void*>(static_cast<const float*>(g) + off)
                         : static_cast<const void*>(static_cast<const uint16_t*>(g) + off);
    std::vector<uint64_t> local(k[t] > 0 ? k[t] : 0);
    int rc = gco_compress_codec(gt, dtype, e + off, n, k[t], block, local.data(), 64, q + qpos,
                                scales + spos, codec);
    if (rc == GCO_ERR_NONFINITE)
      status = rc;
    else if (rc != GCO_OK)
      return rc;
    for (int64_t j = 0; j < k[t]; ++j) {
      uint64_t flat = local[j] + static_cast<uint64_t>(off);
      if (index_bits == 32)
        static_cast<uint32_t*>(idx)[kpos + j] = static_cast<uint32_t>(flat);
      else
        static_cast<uint64_t*>(idx)[kpos + j] = flat;
    }
    kpos += k[t];
    spos += (k[t] + block - 1) / block;
    qpos += gco_num_code_bytes(k[t], block, codec);
  }
  return status;
}

// One error-feedback step on the touched rows of a table-shaped residual (R10). vals: U x D
// gradient values of the touched rows (dtype as in gco_compress), rows: U ascending unique row
// ids in [0, R), e_table: R x D fp32 residual, updated in place on the touched rows only.
// idx receives k table positions (index_bits 64 is required when R * D > 2^32).
int gco_compress_rows(const void* vals, int dtype, float* e_table, const int64_t* rows, int64_t U,
                      int64_t D, int64_t R, int64_t k, int32_t block, void* idx, int32_t index_bits,
                      int8_t* q, float* scales, int32_t codec) {
  if (!vals || !e_table || !rows || !idx) return GCO_ERR_INVALID_ARG;
  if (U < 1 || D < 1 || R < 1 || U > R) return GCO_ERR_INVALID_ARG;
  if (index_bits != 32 && index_bits != 64) return GCO_ERR_INVALID_ARG;
  if (index_bits == 32 && R * D > (int64_t(1) << 32)) return GCO_ERR_INVALID_ARG;
  for (int64_t u = 0; u < U; ++u) {
    if (rows[u] < 0 || rows[u] >= R) return GCO_ERR_INVALID_ARG;
    if (u > 0 && rows[u] <= rows[u - 1]) return GCO_ERR_INVALID_ARG;
  }
  const int64_t m = U * D;
  std::vector<float> ec(static_cast<size_t>(m));
  for (int64_t u = 0; u < U; ++u)
    for (int64_t c = 0; c < D; ++c) ec[u * D + c] = e_table[rows[u] * D + c];
  std::vector<uint64_t> ci(static_cast<size_t>(k > 0 ? k : 1));
  const int rc = gco_compress_codec(vals, dtype, ec.data(), m, k, block, ci.data(), 64, q, scales, codec);
  if (rc == GCO_ERR_INVALID_ARG) return rc;
  for (int64_t j = 0; j < k; ++j) {
    const int64_t c = static_cast<int64_t>(ci[j]);
    const uint64_t pos = static_cast<uint64_t>(rows[c / D] * D + c % D);
    if (index_bits == 32) static_cast<uint32_t*>(idx)[j] = static_cast<uint32_t>(pos);
    else static_cast<uint64_t*>(idx)[j] = pos;
  }
  for (int64_t u = 0; u < U; ++u)
    for (int64_t c = 0; c < D; ++c) e_table[rows[u] * D + c] = ec[u * D + c];
  return rc;
}

int gco_compress_multi(const void* g, int dtype, float* e, const int64_t* offsets,
                       const int64_t* k, int32_t T, int32_t block, void* idx,
                       int32_t index_bits, int8_t* q, float* scales) {
  return gco_compress_multi_codec(g, dtype, e, offsets, k, T, block, idx, index_bits, q, scales, 0);
}

// Sum of W decompressed buffers into a dense vector (Eq. 8 without the 1/P). If `staleness`
// is not null, worker w's decoded value is divided by (1 + staleness[w]) before it is added:
// the damping that Eq. 12 applies to a gradient that is staleness[w] steps late (reading: one
// IEEE fp32 division per entry by the exactly representable 1 + tau, then the fp32 add).
// Buffer w holds kcount[w] entries. If T > 0 the buffers came from
// gco_compress_multi with per-tensor counts ktensor[T] (identical for every
// worker) and the scale of entry j is found per tensor; with T == 0 the scale
// of entry j is scales[j / block].
int gco_decompress_sum_codec(int32_t W, const void* const* idx, const int8_t* const* q,
                             const float* const* scales, const int64_t* kcount, int32_t block,
                             int32_t index_bits, const int64_t* ktensor, int32_t T,
                             const int32_t* staleness, float* out, int64_t n, int32_t codec) {
  if (codec != 0 && codec != 1) return GCO_ERR_INVALID_ARG;
  if (W < 1 || !idx || !q || !scales || !kcount || !out || n <= 0 || block < 1)
    return GCO_ERR_INVALID_ARG;
  if (staleness)
    for (int32_t w = 0; w < W; ++w)
      if (staleness[w] < 0 || staleness[w] > (1 << 24)) return GCO_ERR_INVALID_ARG;
  for (int64_t i = 0; i < n; ++i) out[i] = 0.0f;
  for (int32_t w = 0; w < W; ++w) {
    int64_t t = 0, t_end = (T > 0) ? ktensor[0] : kcount[w], t_begin = 0, s_base = 0, q_base = 0;
    for (int64_t j = 0; j < kcount[w]; ++j) {
      while (T > 0 && j >= t_end) {  // advance to the tensor that owns entry j
        s_base += (t_end - t_begin + block - 1) / block;
        q_base += gco_num_code_bytes(t_end - t_begin, block, codec);
        t_begin = t_end;
        ++t;
        if (t >= T) return GCO_ERR_INVALID_ARG;
        t_end += ktensor[t];
      }
      const float s = scales[w][s_base + (j - t_begin) / block];
      uint64_t i = (index_bits == 32) ? static_cast<const uint32_t*>(idx[w])[j]
                                      : static_cast<const uint64_t*>(idx[w])[j];
      if (i >= static_cast<uint64_t>(n)) return GCO_ERR_INVALID_ARG;
      volatile float d;
      if (codec == 0) {
        d = static_cast<float>(q[w][j]) * s;
      } else {  // sign code: +-s, bit r of the block's bytes
        const int64_t r = (j - t_begin) % block, bb = (j - t_begin) / block;
        const uint8_t byte = reinterpret_cast<const uint8_t*>(q[w])[q_base + bb * ((block + 7) / 8) + r / 8];
        d = ((byte >> (r % 8)) & 1u) ? s : -s;
      }
      if (staleness) {
        const float denom = 1.0f + static_cast<float>(staleness[w]);
        volatile float damped = d / denom;
        d = damped;
      }
      out[i] = out[i] + d;
    }
  }
  return GCO_OK;
}

// Aggregate of W workers' row-sparse buffers over a given set of rows (R10): urows holds Ru
// ascending unique row ids that contain every row any buffer touches; out is Ru x D and
// out[r * D + c] is the worker-ordered fp32 sum of the decoded values at table position
// urows[r] * D + c, exactly as the dense aggregate would hold there. A pair whose row is not
// in urows is an error.
int gco_decompress_sum_rows(int32_t W, const void* const* idx, const int8_t* const* q,
                            const float* const* scales, const int64_t* kcount, int32_t block,
                            int32_t index_bits, const int64_t* urows, int64_t Ru, int64_t D,
                            const int32_t* staleness, float* out, int32_t codec) {
  if (W < 1 || !idx || !kcount || !urows || Ru < 1 || D < 1) return GCO_ERR_INVALID_ARG;
  if (index_bits != 32 && index_bits != 64) return GCO_ERR_INVALID_ARG;
  for (int64_t r = 1; r < Ru; ++r)
    if (urows[r] <= urows[r - 1]) return GCO_ERR_INVALID_ARG;
  std::vector<std::vector<uint64_t>> compact(static_cast<size_t>(W));
  std::vector<const void*> cptr(static_cast<size_t>(W));
  for (int32_t w = 0; w < W; ++w) {
    compact[w].resize(static_cast<size_t>(kcount[w] > 0 ? kcount[w] : 1));
    for (int64_t j = 0; j < kcount[w]; ++j) {
      const uint64_t pos = (index_bits == 32) ? static_cast<const uint32_t*>(idx[w])[j]
                                              : static_cast<const uint64_t*>(idx[w])[j];
      const int64_t row = static_cast<int64_t>(pos / static_cast<uint64_t>(D));
      const int64_t col = static_cast<int64_t>(pos % static_cast<uint64_t>(D));
      const int64_t* it = std::lower_bound(urows, urows + Ru, row);
      if (it == urows + Ru || *it != row) return GCO_ERR_INVALID_ARG;
      compact[w][j] = static_cast<uint64_t>((it - urows) * D + col);
    }
    cptr[w] = compact[w].data();
  }
  return gco_decompress_sum_codec(W, cptr.data(), q, scales, kcount, block, 64, nullptr, 0, staleness, out,
                                  Ru * D, codec);
}

int gco_decompress_sum_weighted(int32_t W, const void* const* idx, const int8_t* const* q,
                                const float* const* scales, const int64_t* kcount, int32_t block,
                                int32_t index_bits, const int64_t* ktensor, int32_t T,
                                const int32_t* staleness, float* out, int64_t n) {
  return gco_decompress_sum_codec(W, idx, q, scales, kcount, block, index_bits, ktensor, T, staleness, out, n,
                                  0);
}

int gco_decompress_sum(int32_t W, const void* const* idx, const int8_t* const* q,
                       const float* const* scales, const int64_t* kcount, int32_t block,
                       int32_t index_bits, const int64_t* ktensor, int32_t T, float* out,
                       int64_t n) {
  return gco_decompress_sum_codec(W, idx, q, scales, kcount, block, index_bits, ktensor, T, nullptr, out, n,
                                  0);
}

// Parameter update with the aggregate (Eq. 9 with g from Eq. 8): theta <- theta - step * S,
// `step` standing for eta / P; two fp32 roundings per entry (product, then difference).
int gco_apply(float* theta, const float* S, float step, int64_t n) {
  if (!theta || !S || n <= 0 || !(step >= 0.0f)) return GCO_ERR_INVALID_ARG;
  for (int64_t i = 0; i < n; ++i) {
    volatile float upd = step * S[i];
    theta[i] = theta[i] - upd;
  }
  return GCO_OK;
}

}  // extern "C"
