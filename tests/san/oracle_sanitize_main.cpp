// Host sanitizer run of the CPU oracle: compiled by tests/test_oracle_sanitize.py together with
// oracle/gc_oracle.cpp under -fsanitize=address,undefined and executed once. It walks every entry
// point of the oracle over ragged sizes, both value codes, both index widths, bf16 input, several
// tensors, the row-sparse step and the aggregates, with output arrays sized exactly (so a write
// one past the end is caught), and checks a few invariants so that the calls cannot be elided.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

extern "C" {
int64_t gco_k_from_density(int64_t n, double density);
int64_t gco_num_code_bytes(int64_t k, int32_t block, int32_t codec);
int gco_compress_codec(const void* g, int dtype, float* e, int64_t n, int64_t k, int32_t block, void* idx,
                       int32_t index_bits, int8_t* q, float* scales, int32_t codec);
int gco_compress_multi_codec(const void* g, int dtype, float* e, const int64_t* offsets, const int64_t* k,
                             int32_t T, int32_t block, void* idx, int32_t index_bits, int8_t* q, float* scales,
                             int32_t codec);
int gco_compress_rows(const void* vals, int dtype, float* e_table, const int64_t* rows, int64_t U, int64_t D,
                      int64_t R, int64_t k, int32_t block, void* idx, int32_t index_bits, int8_t* q,
                      float* scales, int32_t codec);
int gco_decompress_sum_codec(int32_t W, const void* const* idx, const int8_t* const* q, const float* const* scales,
                             const int64_t* kcount, int32_t block, int32_t index_bits, const int64_t* ktensor,
                             int32_t T, const int32_t* staleness, float* out, int64_t n, int32_t codec);
int gco_decompress_sum_rows(int32_t W, const void* const* idx, const int8_t* const* q, const float* const* scales,
                            const int64_t* kcount, int32_t block, int32_t index_bits, const int64_t* urows,
                            int64_t Ru, int64_t D, const int32_t* staleness, float* out, int32_t codec);
int gco_apply(float* theta, const float* S, float step, int64_t n);
}

namespace {

uint64_t state = 0x243F6A8885A308D3ull;
uint32_t next_u32() {  // splitmix64, upper half
  uint64_t z = (state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return (uint32_t)((z ^ (z >> 31)) >> 32);
}
float next_val() {  // a few exact ties, zeros of both signs, and a wide spread
  const uint32_t r = next_u32();
  if (r % 11 == 0) return 0.0f;
  if (r % 13 == 0) return -0.0f;
  if (r % 7 == 0) return 0.5f;
  const float m = (float)(r >> 8) / 16777216.0f - 0.5f;
  return m * ((r & 1u) ? 1e-3f : 40.0f);
}

#define CHECK(c)                                                     \
  do {                                                               \
    if (!(c)) {                                                      \
      std::fprintf(stderr, "check failed line %d: %s\n", __LINE__, #c); \
      std::exit(3);                                                  \
    }                                                                \
  } while (0)

struct Buf {
  std::vector<uint32_t> i32;
  std::vector<uint64_t> i64;
  std::vector<int8_t> q;
  std::vector<float> s;
};

void flat_case(int64_t n, int64_t k, int32_t block, int bits, int codec, int dtype) {
  std::vector<float> g32(n), e(n);
  std::vector<uint16_t> g16(n);
  for (int64_t i = 0; i < n; ++i) {
    g32[i] = next_val();
    union { float f; uint32_t u; } c;
    c.f = g32[i];
    g16[i] = (uint16_t)(c.u >> 16);
    e[i] = next_val() * 0.25f;
  }
  Buf b;
  b.i32.resize(bits == 32 ? k : 0);
  b.i64.resize(bits == 64 ? k : 0);
  b.q.resize(gco_num_code_bytes(k, block, codec));
  b.s.resize((k + block - 1) / block);
  void* ip = bits == 32 ? (void*)b.i32.data() : (void*)b.i64.data();
  const void* gp = dtype == 0 ? (const void*)g32.data() : (const void*)g16.data();
  CHECK(gco_compress_codec(gp, dtype, e.data(), n, k, block, ip, bits, b.q.data(), b.s.data(), codec) == 0);
  for (int64_t j = 1; j < k; ++j)
    CHECK(bits == 32 ? b.i32[j] > b.i32[j - 1] : b.i64[j] > b.i64[j - 1]);
  // aggregate of three copies, with and without staleness
  const void* ia[3] = {ip, ip, ip};
  const int8_t* qa[3] = {b.q.data(), b.q.data(), b.q.data()};
  const float* sa[3] = {b.s.data(), b.s.data(), b.s.data()};
  const int64_t kc[3] = {k, k, k};
  const int32_t stale[3] = {0, 2, 5};
  std::vector<float> out(n), theta(n, 1.0f);
  CHECK(gco_decompress_sum_codec(3, ia, qa, sa, kc, block, bits, nullptr, 0, nullptr, out.data(), n, codec) == 0);
  CHECK(gco_decompress_sum_codec(3, ia, qa, sa, kc, block, bits, nullptr, 0, stale, out.data(), n, codec) == 0);
  CHECK(gco_apply(theta.data(), out.data(), 0.125f, n) == 0);
}

void multi_case(int codec) {
  const int64_t sizes[] = {1, 5, 768, 1025, 33, 4097, 2};
  const int32_t T = 7, block = 16;
  std::vector<int64_t> off(T + 1, 0), ks(T);
  int64_t ktot = 0, stot = 0, qtot = 0;
  for (int t = 0; t < T; ++t) {
    off[t + 1] = off[t] + sizes[t];
    ks[t] = gco_k_from_density(sizes[t], 0.05);
    ktot += ks[t];
    stot += (ks[t] + block - 1) / block;
    qtot += gco_num_code_bytes(ks[t], block, codec);
  }
  const int64_t n = off[T];
  std::vector<float> g(n), e(n);
  for (int64_t i = 0; i < n; ++i) { g[i] = next_val(); e[i] = next_val(); }
  std::vector<uint32_t> idx(ktot);
  std::vector<int8_t> q(qtot);
  std::vector<float> s(stot);
  CHECK(gco_compress_multi_codec(g.data(), 0, e.data(), off.data(), ks.data(), T, block, idx.data(), 32, q.data(),
                                 s.data(), codec) == 0);
  const void* ia[2] = {idx.data(), idx.data()};
  const int8_t* qa[2] = {q.data(), q.data()};
  const float* sa[2] = {s.data(), s.data()};
  const int64_t kc[2] = {ktot, ktot};
  std::vector<float> out(n);
  CHECK(gco_decompress_sum_codec(2, ia, qa, sa, kc, block, 32, ks.data(), T, nullptr, out.data(), n, codec) == 0);
}

void rows_case(int codec, int bits) {
  const int64_t R = 97, D = 12, U = 9, block = 8;
  const int64_t rows[U] = {0, 3, 4, 17, 40, 41, 42, 90, 96};
  const int64_t k = 23;
  std::vector<float> vals(U * D), table(R * D);
  for (auto& v : vals) v = next_val();
  for (auto& v : table) v = next_val() * 0.1f;
  std::vector<uint32_t> i32(bits == 32 ? k : 0);
  std::vector<uint64_t> i64(bits == 64 ? k : 0);
  std::vector<int8_t> q(gco_num_code_bytes(k, block, codec));
  std::vector<float> s((k + block - 1) / block);
  void* ip = bits == 32 ? (void*)i32.data() : (void*)i64.data();
  CHECK(gco_compress_rows(vals.data(), 0, table.data(), rows, U, D, R, k, (int32_t)block, ip, bits, q.data(), s.data(),
                          codec) == 0);
  const void* ia[1] = {ip};
  const int8_t* qa[1] = {q.data()};
  const float* sa[1] = {s.data()};
  const int64_t kc[1] = {k};
  std::vector<float> out(U * D);
  CHECK(gco_decompress_sum_rows(1, ia, qa, sa, kc, (int32_t)block, bits, rows, U, D, nullptr, out.data(), codec) == 0);
}

}  // namespace

int main() {
  const int64_t ns[] = {1, 2, 63, 64, 65, 1000, 4097, 20011};
  for (int64_t n : ns)
    for (int codec = 0; codec < 2; ++codec)
      for (int bits = 32; bits <= 64; bits += 32) {
        const int64_t kk[] = {1, (n + 9) / 10, n};
        for (int64_t k : kk)
          for (int32_t block : {1, 7, 256}) flat_case(n, k, block, bits, codec, (int)((n + k) & 1));
      }
  for (int codec = 0; codec < 2; ++codec) {
    multi_case(codec);
    rows_case(codec, 32);
    rows_case(codec, 64);
  }
  // argument errors return without touching anything
  float one = 1.0f;
  uint32_t i1 = 0;
  int8_t q1 = 0;
  CHECK(gco_compress_codec(&one, 0, &one, 1, 2, 1, &i1, 32, &q1, &one, 0) != 0);
  CHECK(gco_compress_codec(&one, 0, &one, 1, 1, 0, &i1, 32, &q1, &one, 0) != 0);
  CHECK(gco_compress_codec(nullptr, 0, &one, 1, 1, 1, &i1, 32, &q1, &one, 0) != 0);
  std::puts("oracle sanitizer run: ok");
  return 0;
}
