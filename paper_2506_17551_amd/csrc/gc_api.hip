// Host side of libgradcomp: argument checks, the per-shape plan, workspace, launch order
// and the C ABI declared in include/gradcomp.h.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/gradcomp.h"
#include "gc_internal.h"

using namespace gc;

namespace {

struct DevBuf {
  void* p = nullptr;
  size_t bytes = 0;
};

struct Plan {  // everything that depends only on (offsets, k, block)
  std::vector<int64_t> offsets, k;
  int32_t block = 0, codec = 0;
  std::vector<TensorDesc> td;
  int32_t cap = 0;            // candidate slots per group
  int32_t slot_stride = 16;   // records reserved per group: 8, or a multiple of 16
  int32_t gather_team = 1;    // lanes that copy one group's candidates
  int64_t ngroups = 0, nsgran = 0, cand_total_cap = 0, ktotal = 0, stotal = 0, max_chunks = 0;
  int64_t n_sampled = 0, est_chunks = 0;
  int64_t n_small = 0;      // tensors finished by one workgroup (k_finish)
  int64_t n_general = 0;    // tensors that take the chain of grid-wide kernels
  std::vector<GroupRec> recs;  // one per group, only when there are several tensors
  DevBuf td_dev, recs_dev;
};

struct DecPlan {  // per-tensor prefix tables for multi-tensor decompress
  std::vector<int64_t> k;
  int32_t block = 0, codec = 0;
  DevBuf kprefix, sprefix, qprefix;
};

struct EventPair {
  hipEvent_t a, b;
  int32_t id;
};

}  // namespace

struct gc_ctx {
  int device = 0;
  std::vector<Plan*> plans;
  std::vector<DecPlan*> dplans;
  // workspace (sized for the largest plan seen)
  DevBuf rows_e, rows_idx;  // compact residual and compact positions of a row-sparse step
  DevBuf rows_cidx;         // compact positions of all workers' pairs (aggregate over a row list)
  DevBuf ts, shist, hist, grp_cnt, grp_part, grp_off, tg_base, slots, cand_val, cand_idx, ch_gt,
      ch_eq, ch_part_gt, ch_part_eq, ch_goff, ch_eoff, tb_g, tb_e, totals, kept_val, flags;
  DevBuf dec_rec, dec_tile_start;  // aggregate: packed pair records, first record of every tile
  uint32_t* host_flags = nullptr;  // pinned
  TensorState* host_ts = nullptr;  // pinned copy for gc_last_stats
  size_t host_ts_cap = 0;
  Plan* single = nullptr;  // plan of the last single-tensor call: rebuilt per call on the host, never uploaded
  const Plan* last_plan = nullptr;
  int64_t last_dense_tensors = 0;  // tensors of the last compress call when it took the dense coder
  int64_t opt_main_lds_pad = 16384;  // dynamic LDS of the streaming pass: at most 8 workgroups per CU
  int64_t opt_dense_wave_block = 1024;  // dense coder: blocks up to this size are held by one wavefront
  int64_t opt_dense_lds_pad = -1;       // dense coder: dynamic LDS per workgroup (occupancy bound); -1: by shape
  int64_t opt_dec_large_tile = -1;      // aggregate: 16384-float tiles (1), 4096-float tiles (0), or by shape (-1)
  int64_t opt_dec_fused_tile = -1;      // one-kernel aggregate: the shape for thin tiles (0), for crowded ones (1), by filling (-1)
  int64_t opt_dec_fused = -1;           // aggregate: the one-kernel route without the record stream (1), the two-kernel route (0), by filling (-1)
  int64_t opt_apply_dense_min = 128;    // fused apply: tiles with at least this many records per 4096 floats are rewritten whole
  // profiling
  int prof = 0;  // 0 off, 1 every kernel, 2 only the streaming pass
  std::vector<EventPair> ev_used, ev_free;
};

// ---- scratch of the entry point that allocates nothing --------------------------
// gc_decompress_sum_static keeps its record stream and tile starts in this array
// instead of the context's workspace. Every device the library runs on holds its own copy at its own
// address; the name below is only a host-side handle, so host code asks the runtime for the device
// address once per device (in gc_create, with that device current) and uses that pointer from then on.
constexpr size_t kStaticScratchBytes = (size_t)GC_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, once looked up
static std::mutex g_scratch_mu;

namespace {

#define GC_HIP(expr)                          \
  do {                                        \
    if ((expr) != hipSuccess) {               \
      (void)hipGetLastError();                \
      return GC_ERR_DEVICE;                   \
    }                                         \
  } while (0)

gc_status ensure(DevBuf& b, size_t bytes) {
  if (bytes <= b.bytes) return GC_OK;
  if (b.p) {
    if (hipDeviceSynchronize() != hipSuccess) return GC_ERR_DEVICE;
    if (hipFree(b.p) != hipSuccess) return GC_ERR_DEVICE;
    b.p = nullptr;
    b.bytes = 0;
  }
  size_t want = bytes + bytes / 8 + 256;
  if (hipMalloc(&b.p, want) != hipSuccess) {
    (void)hipGetLastError();
    b.p = nullptr;
    return GC_ERR_WORKSPACE;
  }
  b.bytes = want;
  return GC_OK;
}

void release(DevBuf& b) {
  if (b.p) (void)hipFree(b.p);
  b.p = nullptr;
  b.bytes = 0;
}

int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// ---- plan ------------------------------------------------------------------
// Tensors large and sparse enough get their candidates from a sampled threshold in
// the single streaming pass; the rest are selected from the dense residual.
constexpr int64_t kMinSampledN = 1 << 15;
constexpr int64_t kMinSampledK = 32;
constexpr int64_t kMaxDensityInv = 8;  // sampled only if k * 8 <= n
#ifndef GC_MAX_SAMPLE_STRIDE
#define GC_MAX_SAMPLE_STRIDE 1024
#endif
constexpr int64_t kMaxSampleStride = GC_MAX_SAMPLE_STRIDE;

int64_t code_bytes(int64_t k, int32_t block, int32_t codec) {
  if (k <= 0 || block < 1) return 0;
  if (codec == GC_CODEC_INT8) return k;
  return (k / block) * ((block + 7) / 8) + (k % block + 7) / 8;
}

Plan* build_plan(const int64_t* offsets, const int64_t* k, int32_t T, int32_t block, int32_t codec) {
  Plan* P = new (std::nothrow) Plan();
  if (!P) return nullptr;
  P->offsets.assign(offsets, offsets + T + 1);
  P->k.assign(k, k + T);
  P->block = block;
  P->codec = codec;
  P->td.resize(T);
  int64_t grp = 0, kp = 0, sp = 0, sg = 0, cb = 0, est = 0, qp = 0;
  double max_lambda = 0.0;
  for (int32_t t = 0; t < T; ++t) {
    TensorDesc& d = P->td[t];
    std::memset(&d, 0, sizeof(d));
    d.off = offsets[t];
    d.n = offsets[t + 1] - offsets[t];
    d.k = k[t];
    d.kprefix = kp;
    d.sprefix = sp;
    d.qprefix = qp;
    qp += code_bytes(d.k, block, codec);
    d.group_begin = grp;
    // Groups lie on the grid of the FLAT buffer (boundaries at multiples of 4 elements from its
    // start), so that only a tensor's first group can start unaligned: one odd-sized tensor must
    // not push every later tensor onto the scalar path. With several tensors the first group is
    // shortened by `group_shift` = off % 4 elements.
    d.group_shift = T > 1 ? (int32_t)(d.off % 4) : 0;
    d.ngroups = (d.group_shift + d.n + kGroup - 1) / kGroup;
    grp += d.ngroups;
    P->max_chunks += (d.group_shift + d.n + kChunkElems - 1) / kChunkElems;
    kp += d.k;
    sp += (d.k + block - 1) / block;
    d.sgran_begin = sg;
    d.cand_begin = cb;
    const bool sampled = d.n >= kMinSampledN && d.k >= kMinSampledK && d.k * kMaxDensityInv <= d.n;
    d.mode = sampled ? kSampled : kDense;
    d.small = (sampled ? (d.n <= kSmallMaxN && d.k <= kSmallMaxK) : d.n <= kSmallMaxDenseN) ? 1 : 0;
    if (d.small) P->n_small++; else P->n_general++;
    if (sampled) {
      // sample about 32 expected winners, between 1/256 and 1/4 of the data: a thin sample only
      // makes the candidate list a little longer, and candidates are cheap (and a sample that
      // undershoots only sends the tensor down the dense route, never changes the result)
      double f = 32.0 / (double)d.k;
      // where the tensor is small in absolute terms a denser sample (up to 65536 elements, about
      // 1024 expected winners) costs nothing and halves the candidate list, which the one
      // workgroup that finishes a small tensor then holds in LDS
      f = std::max(f, std::min(1024.0 / (double)d.k, 65536.0 / (double)d.n));
      f = std::min(0.25, std::max(1.0 / 256.0, f));
      int64_t stride = std::max<int64_t>(4, std::min<int64_t>(256, (int64_t)std::floor(1.0 / f)));
      // a very large k leaves thousands of winners in a thinner sample still (at least 4096 expected)
      if (d.k / 4096 > stride) stride = std::min<int64_t>(kMaxSampleStride, d.k / 4096);
      d.sample_stride = (int32_t)stride;
      d.nsgran = (d.n / kSampleGranule) / stride;  // whole granules only; >= 1: k * 8 <= n bounds the stride by n / 256
      sg += round_up(d.nsgran, 4);
      const double m = (double)d.nsgran * kSampleGranule;
      const double ks = (double)d.k * m / (double)d.n;
      // the threshold must leave at least k entries above it: cover the expected sample count
      // of winners plus six standard deviations
      const double target = std::ceil(ks + 6.0 * std::sqrt(ks) + 8.0);
      d.sample_target = (uint32_t)std::min<double>(target, 4.0e9);
      max_lambda = std::max(max_lambda, target / m * (double)kGroup);  // candidates expected per group
      d.cand_cap = std::min<int64_t>(d.n, 8 * d.k + 4096);  // room for ties around the threshold before the dense route
      cb += round_up(d.cand_cap, 4);  // every region starts 16-byte aligned (128-bit loads)
      est += (std::min<int64_t>(d.cand_cap, 2 * d.k) + kChunkElems - 1) / kChunkElems + 1;
      P->n_sampled++;
    } else {
      est += (d.group_shift + d.n + kChunkElems - 1) / kChunkElems;
    }
  }
  if (T > 1) {
    P->recs.resize((size_t)grp);
    for (int32_t t = 0; t < T; ++t) {
      const TensorDesc& d = P->td[t];
      for (int64_t lg = 0; lg < d.ngroups; ++lg) {
        GroupRec& r = P->recs[(size_t)(d.group_begin + lg)];
        const int64_t first = std::max<int64_t>(0, lg * kGroup - d.group_shift);  // inside the tensor
        const int64_t next = std::min<int64_t>(d.n, (lg + 1) * kGroup - d.group_shift);
        r.start = d.off + first;
        r.len = (int32_t)(next - first);
        r.tensor = (uint32_t)t | (d.mode == kSampled ? 0x80000000u : 0u);
      }
    }
  }
  P->ngroups = grp;
  P->nsgran = sg;
  P->cand_total_cap = cb;
  P->ktotal = kp;
  P->stotal = sp;
  P->est_chunks = est;
  // a group that gets more candidates than slots is re-read by the gather, so the slots only
  // need to cover the ordinary spread of the count
  const double cap = std::ceil(max_lambda + 5.0 * std::sqrt(max_lambda) + 1.0);
  P->cap = (int32_t)std::min<double>((double)round_up((int64_t)cap, kSlotLine), (double)kGroup);
  if (cap <= kSlotLine / 2) P->cap = kSlotLine / 2;  // half a line per group is enough (7B at 0.1 %: 1.15 expected)
  if (P->n_sampled == 0) P->cap = kSlotLine;
  P->cap = std::min(P->cap, 4096);  // the LDS staging holds cap records (at most 32 KB)
  P->slot_stride = P->cap;           // whole 128-byte lines of records, or half a line
  // measured: one lane per group is faster up to ~6 candidates per group, 16 lanes from ~11 on
  P->gather_team = max_lambda >= 8.0 ? 16 : 1;
  return P;
}

bool same_plan(const Plan* P, const int64_t* offsets, const int64_t* k, int32_t T, int32_t block,
               int32_t codec) {
  return P->block == block && P->codec == codec && (int32_t)P->k.size() == T &&
         std::memcmp(P->offsets.data(), offsets, sizeof(int64_t) * (T + 1)) == 0 &&
         std::memcmp(P->k.data(), k, sizeof(int64_t) * T) == 0;
}

// What a compress call needs of the context's workspace, in entries of each array.
struct Need {
  size_t T = 0, ngroups = 0, slot_records = 0, cand = 0, max_chunks = 0, ktotal = 0, stotal = 0;
  bool sampled = false;
};

Need need_of(const Plan* P) {
  Need nd;
  nd.T = P->td.size();
  nd.ngroups = (size_t)P->ngroups;
  nd.sampled = P->n_sampled > 0;
  nd.slot_records = nd.sampled ? (size_t)P->ngroups * (size_t)P->slot_stride : 0;
  nd.cand = nd.sampled ? (size_t)P->cand_total_cap : 0;
  nd.max_chunks = (size_t)P->max_chunks;
  nd.ktotal = (size_t)P->ktotal;
  nd.stotal = (size_t)P->stotal;
  return nd;
}

// Grows the workspace to what `nd` needs. Growing an array waits for the device, frees and allocates;
// once the arrays are large enough (gc_reserve, or an earlier call of the same size) this does nothing.
gc_status ensure_workspace(gc_ctx* ctx, const Need& nd) {
  const size_t T = nd.T, ng = nd.ngroups, nent = nd.max_chunks * 4;
  const size_t ngp = (ng + kScanBlock - 1) / kScanBlock, ncp = (nent + kScanBlock - 1) / kScanBlock;
  gc_status st = ensure(ctx->ts, sizeof(TensorState) * T);
  if (st == GC_OK) {  // the sample histograms start zeroed too, and the threshold kernel leaves them so
    const void* before = ctx->shist.p;
    st = ensure(ctx->shist, sizeof(unsigned long long) * T * kSampleBins);
    if (st == GC_OK && ctx->shist.p != before && hipMemset(ctx->shist.p, 0, ctx->shist.bytes) != hipSuccess)
      st = GC_ERR_DEVICE;
  }
  if (st == GC_OK) {  // the select histograms must start zeroed; every call leaves them zeroed again
    const void* before = ctx->hist.p;
    st = ensure(ctx->hist, sizeof(unsigned long long) * T * kSelBins);
    if (st == GC_OK && ctx->hist.p != before && hipMemset(ctx->hist.p, 0, ctx->hist.bytes) != hipSuccess)
      st = GC_ERR_DEVICE;
  }
  if (st == GC_OK) st = ensure(ctx->grp_cnt, sizeof(uint32_t) * ng);
  if (st == GC_OK) st = ensure(ctx->grp_part, sizeof(unsigned long long) * ngp);
  if (st == GC_OK) st = ensure(ctx->grp_off, sizeof(long long) * ng);
  if (st == GC_OK) st = ensure(ctx->tg_base, sizeof(long long) * (T + 1));
  if (nd.sampled) {
    if (st == GC_OK) st = ensure(ctx->slots, sizeof(uint2) * nd.slot_records);
    if (st == GC_OK) st = ensure(ctx->cand_val, sizeof(float) * nd.cand);
    if (st == GC_OK) st = ensure(ctx->cand_idx, sizeof(long long) * nd.cand);
  }
  if (st == GC_OK) st = ensure(ctx->ch_gt, sizeof(uint32_t) * nent);
  if (st == GC_OK) st = ensure(ctx->ch_eq, sizeof(uint32_t) * nent);
  if (st == GC_OK) st = ensure(ctx->ch_part_gt, sizeof(unsigned long long) * ncp);
  if (st == GC_OK) st = ensure(ctx->ch_part_eq, sizeof(unsigned long long) * ncp);
  if (st == GC_OK) st = ensure(ctx->ch_goff, sizeof(long long) * nent);
  if (st == GC_OK) st = ensure(ctx->ch_eoff, sizeof(long long) * nent);
  if (st == GC_OK) st = ensure(ctx->tb_g, sizeof(long long) * T);
  if (st == GC_OK) st = ensure(ctx->tb_e, sizeof(long long) * T);
  if (st == GC_OK) st = ensure(ctx->totals, sizeof(long long) * 4);
  if (st == GC_OK) st = ensure(ctx->kept_val, sizeof(float) * nd.ktotal);
  if (st == GC_OK && ctx->host_ts_cap < T) {
    if (ctx->host_ts) (void)hipHostFree(ctx->host_ts);
    ctx->host_ts = nullptr;
    ctx->host_ts_cap = 0;
    if (hipHostMalloc((void**)&ctx->host_ts, sizeof(TensorState) * T, hipHostMallocDefault) != hipSuccess)
      st = GC_ERR_WORKSPACE;
    else
      ctx->host_ts_cap = T;
  }
  return st;
}

// A single-tensor call needs no cache entry and no upload: its plan is a few numbers, rebuilt on
// the host for every call and handed to the kernels by argument. A shape that changes from call to
// call (the touched rows of an embedding gradient) therefore costs nothing extra.
gc_status get_single_plan(gc_ctx* ctx, const int64_t* offsets, const int64_t* k, int32_t block, int32_t codec,
                          Plan** out) {
  Plan* P = build_plan(offsets, k, 1, block, codec);
  if (!P) return GC_ERR_WORKSPACE;
  if (ctx->last_plan == ctx->single) ctx->last_plan = nullptr;
  delete ctx->single;
  ctx->single = P;
  const gc_status st = ensure_workspace(ctx, need_of(P));
  if (st != GC_OK) return st;
  *out = P;
  return GC_OK;
}

gc_status get_plan(gc_ctx* ctx, const int64_t* offsets, const int64_t* k, int32_t T, int32_t block,
                   int32_t codec, Plan** out) {
  for (size_t i = 0; i < ctx->plans.size(); ++i) {
    if (same_plan(ctx->plans[i], offsets, k, T, block, codec)) {
      Plan* P = ctx->plans[i];
      if (i != 0) {  // keep the most recent first
        ctx->plans.erase(ctx->plans.begin() + i);
        ctx->plans.insert(ctx->plans.begin(), P);
      }
      *out = P;
      return GC_OK;
    }
  }
  Plan* P = build_plan(offsets, k, T, block, codec);
  if (!P) return GC_ERR_WORKSPACE;
  gc_status st = ensure(P->td_dev, sizeof(TensorDesc) * T);
  if (st == GC_OK && hipMemcpy(P->td_dev.p, P->td.data(), sizeof(TensorDesc) * T, hipMemcpyHostToDevice) != hipSuccess)
    st = GC_ERR_DEVICE;
  if (st == GC_OK && !P->recs.empty()) {
    st = ensure(P->recs_dev, sizeof(GroupRec) * P->recs.size());
    if (st == GC_OK && hipMemcpy(P->recs_dev.p, P->recs.data(), sizeof(GroupRec) * P->recs.size(),
                                 hipMemcpyHostToDevice) != hipSuccess)
      st = GC_ERR_DEVICE;
    std::vector<GroupRec>().swap(P->recs);
  }
  if (st == GC_OK) st = ensure_workspace(ctx, need_of(P));
  if (st != GC_OK) {
    release(P->td_dev);
    release(P->recs_dev);
    delete P;
    return st;
  }
  ctx->plans.insert(ctx->plans.begin(), P);
  while (ctx->plans.size() > 8) {
    Plan* old = ctx->plans.back();
    ctx->plans.pop_back();
    if (ctx->last_plan == old) ctx->last_plan = nullptr;
    (void)hipDeviceSynchronize();
    release(old->td_dev);
    release(old->recs_dev);
    delete old;
  }
  *out = P;
  return GC_OK;
}

// ---- profiling -------------------------------------------------------------
struct Scope {  // records an event pair around one launch when profiling is on
  gc_ctx* c;
  hipStream_t s;
  EventPair ev;
  bool on;
  Scope(gc_ctx* ctx, int32_t id, hipStream_t st)
      : c(ctx), s(st), on(ctx && (ctx->prof == 1 || (ctx->prof == 2 && id == kKMain))) {
    if (!on) return;
    if (!c->ev_free.empty()) {
      ev = c->ev_free.back();
      c->ev_free.pop_back();
    } else if (hipEventCreate(&ev.a) != hipSuccess || hipEventCreate(&ev.b) != hipSuccess) {
      on = false;
      return;
    }
    ev.id = id;
    (void)hipEventRecord(ev.a, s);
  }
  ~Scope() {
    if (!on) return;
    (void)hipEventRecord(ev.b, s);
    c->ev_used.push_back(ev);
  }
};

gc_status launch_status() { return hipGetLastError() == hipSuccess ? GC_OK : GC_ERR_DEVICE; }

gc_status compress_impl(gc_ctx* ctx, const void* grad, gc_dtype dtype, float* residual,
                        const int64_t* offsets, const int64_t* k, int32_t T, int32_t block,
                        const gc_buf* out, void* hip_stream) {
  if (!ctx || !grad || !residual || !offsets || !k || !out) return GC_ERR_INVALID_ARG;
  if (T < 1 || block < 1) return GC_ERR_INVALID_ARG;
  if (dtype != GC_F32 && dtype != GC_BF16) return GC_ERR_INVALID_ARG;
  if (!out->indices || !out->q || !out->scales) return GC_ERR_INVALID_ARG;
  if (offsets[0] != 0) return GC_ERR_INVALID_ARG;
  int64_t ktotal = 0;
  for (int32_t t = 0; t < T; ++t) {
    const int64_t nt = offsets[t + 1] - offsets[t];
    if (nt <= 0 || k[t] < 1 || k[t] > nt) return GC_ERR_INVALID_ARG;
    ktotal += k[t];
  }
  const int64_t n = offsets[T];
  if (ktotal >= (int64_t(1) << 32)) return GC_ERR_UNSUPPORTED;
  if (out->n != n || out->k != ktotal || out->block != block) return GC_ERR_INVALID_ARG;
  if (out->index_bits != 32 && out->index_bits != 64) return GC_ERR_INVALID_ARG;
  if (out->index_bits == 32 && n > (int64_t(1) << 32)) return GC_ERR_INVALID_ARG;
  if (out->codec != GC_CODEC_INT8 && out->codec != GC_CODEC_SIGN1) return GC_ERR_INVALID_ARG;
  if (out->reserved_ != 0) return GC_ERR_INVALID_ARG;
  if (out->codec == GC_CODEC_SIGN1 && block > 8192) return GC_ERR_UNSUPPORTED;
  const size_t gsz = dtype == GC_F32 ? 4 : 2;
  if ((reinterpret_cast<uintptr_t>(grad) % gsz) || (reinterpret_cast<uintptr_t>(residual) % 4) ||
      (reinterpret_cast<uintptr_t>(out->scales) % 4) ||
      (reinterpret_cast<uintptr_t>(out->indices) % (out->index_bits / 8)))
    return GC_ERR_INVALID_ARG;

  GC_HIP(hipSetDevice(ctx->device));
  if (T == 1 && k[0] == n && block <= kDenseMaxBlock) {
    // every entry is kept: no selection, the one-pass dense coder writes the same result
    hipStream_t ds = (hipStream_t)hip_stream;
    {
      Scope sc(ctx, kKDense, ds);
      launch_dense(grad, (int)dtype, residual, n, block, out->codec, out->q, out->scales, out->indices,
                   out->index_bits, (uint32_t*)ctx->flags.p, (int)ctx->opt_dense_wave_block,
                   (int)ctx->opt_dense_lds_pad, ds);
    }
    ctx->last_plan = nullptr;
    ctx->last_dense_tensors = 1;
    return launch_status();
  }
  ctx->last_dense_tensors = 0;
  Plan* P = nullptr;
  gc_status st = T == 1 ? get_single_plan(ctx, offsets, k, block, out->codec, &P)
                        : get_plan(ctx, offsets, k, T, block, out->codec, &P);
  if (st != GC_OK) return st;
  if (xcd_run_grid(P->ngroups) >= (int64_t(1) << 31)) return GC_ERR_UNSUPPORTED;

  Workspace ws;
  std::memset(&ws, 0, sizeof(ws));
  if (T == 1) {
    ws.td = nullptr;
    ws.td1 = P->td[0];
  } else {
    ws.td = (const TensorDesc*)P->td_dev.p;
  }
  ws.recs = (const GroupRec*)P->recs_dev.p;
  ws.n_single = offsets[T];
  ws.ts = (TensorState*)ctx->ts.p;
  ws.shist = (unsigned long long*)ctx->shist.p;
  ws.hist = (unsigned long long*)ctx->hist.p;
  ws.grp_cnt = (uint32_t*)ctx->grp_cnt.p;
  ws.grp_part = (unsigned long long*)ctx->grp_part.p;
  ws.grp_off = (long long*)ctx->grp_off.p;
  ws.tg_base = (long long*)ctx->tg_base.p;
  ws.slots = (uint2*)ctx->slots.p;
  ws.slot_stride = P->slot_stride;
  ws.cand_val = (float*)ctx->cand_val.p;
  ws.cand_idx = (long long*)ctx->cand_idx.p;
  ws.ch_gt = (uint32_t*)ctx->ch_gt.p;
  ws.ch_eq = (uint32_t*)ctx->ch_eq.p;
  ws.ch_part_gt = (unsigned long long*)ctx->ch_part_gt.p;
  ws.ch_part_eq = (unsigned long long*)ctx->ch_part_eq.p;
  ws.ch_goff = (long long*)ctx->ch_goff.p;
  ws.ch_eoff = (long long*)ctx->ch_eoff.p;
  ws.tb_g = (long long*)ctx->tb_g.p;
  ws.tb_e = (long long*)ctx->tb_e.p;
  ws.totals = (long long*)ctx->totals.p;
  ws.kept_val = (float*)ctx->kept_val.p;
  ws.nblocks = P->stotal;
  ws.flags = (uint32_t*)ctx->flags.p;
  ws.T = T;
  ws.block = block;
  ws.cap = P->cap;
  ws.gather_team = P->gather_team;
  ws.ngroups = P->ngroups;
  ws.nsgran = P->nsgran;
  ws.max_chunks = P->max_chunks;
  ws.max_chunk_wgs = (int32_t)std::min<int64_t>(P->max_chunks, 1 << 20);
  ws.main_lds_pad = (int32_t)ctx->opt_main_lds_pad;
  OutBuf ob{out->indices, out->q, out->scales, out->index_bits, block, out->codec};
  hipStream_t s = (hipStream_t)hip_stream;
  const bool any_sampled = P->n_sampled > 0;

  const bool any_general = P->n_general > 0;
  if (any_sampled) {
    { Scope sc(ctx, kKSample, s); launch_sample(ws, grad, (int)dtype, residual, s); }
    { Scope sc(ctx, kKSampleThresh, s); launch_sample_thresh(ws, s); }
  }
  { Scope sc(ctx, kKMain, s); launch_main(ws, grad, (int)dtype, residual, s); }
  // small tensors: one workgroup each does everything that is left, in one launch
  if (P->n_small > 0) { Scope sc(ctx, kKFinish, s); launch_finish(ws, residual, ob, s); }
  if (any_general) {
    if (any_sampled) {
      { Scope sc(ctx, kKGroupSums, s); launch_group_sums(ws, s); }
      { Scope sc(ctx, kKGroupScan, s); launch_group_scan(ws, s); }
    }
    // (a single sampled tensor is routed by the last block of k_group_scan)
    if (!(T == 1 && any_sampled)) { Scope sc(ctx, kKRoute, s); launch_route(ws, s); }
    if (any_sampled) { Scope sc(ctx, kKGather, s); launch_gather(ws, residual, s); }
    for (int level = 0; level < kSelLevels; ++level) {
      { Scope sc(ctx, kKHist, s); launch_hist(ws, level, residual, s); }
      { Scope sc(ctx, kKSelectScan, s); launch_select_scan(ws, level, s); }
    }
    { Scope sc(ctx, kKCount, s); launch_count(ws, residual, s); }
    { Scope sc(ctx, kKChunkSums, s); launch_chunk_sums(ws, s); }
    { Scope sc(ctx, kKChunkScan, s); launch_chunk_scan(ws, s); }
    { Scope sc(ctx, kKEmit, s); launch_emit(ws, residual, ob, s); }
  }
  // the grid-wide coder: every block of the sign code, and the int8 code of the general tensors
  if (any_general || out->codec == GC_CODEC_SIGN1) { Scope sc(ctx, kKQuant, s); launch_quant(ws, residual, ob, P->ktotal, s); }
  ctx->last_plan = P;
  return launch_status();
}

gc_status get_dec_plan(gc_ctx* ctx, const int64_t* k, int32_t T, int32_t block, int32_t codec,
                       DecPlan** out) {
  for (size_t i = 0; i < ctx->dplans.size(); ++i) {
    DecPlan* D = ctx->dplans[i];
    if (D->block == block && D->codec == codec && (int32_t)D->k.size() == T && std::memcmp(D->k.data(), k, sizeof(int64_t) * T) == 0) {
      if (i != 0) {  // keep the most recently used first: the last entry is the one evicted
        ctx->dplans.erase(ctx->dplans.begin() + i);
        ctx->dplans.insert(ctx->dplans.begin(), D);
      }
      *out = D;
      return GC_OK;
    }
  }
  DecPlan* D = new (std::nothrow) DecPlan();
  if (!D) return GC_ERR_WORKSPACE;
  D->k.assign(k, k + T);
  D->block = block;
  D->codec = codec;
  std::vector<long long> kp(T + 1), sp(T + 1), qp(T + 1);
  kp[0] = sp[0] = qp[0] = 0;
  for (int32_t t = 0; t < T; ++t) {
    kp[t + 1] = kp[t] + k[t];
    sp[t + 1] = sp[t] + (k[t] + block - 1) / block;
    qp[t + 1] = qp[t] + code_bytes(k[t], block, codec);
  }
  gc_status st = ensure(D->kprefix, sizeof(long long) * (T + 1));
  if (st == GC_OK) st = ensure(D->sprefix, sizeof(long long) * (T + 1));
  if (st == GC_OK) st = ensure(D->qprefix, sizeof(long long) * (T + 1));
  if (st == GC_OK && hipMemcpy(D->qprefix.p, qp.data(), sizeof(long long) * (T + 1), hipMemcpyHostToDevice) != hipSuccess)
    st = GC_ERR_DEVICE;
  if (st == GC_OK && (hipMemcpy(D->kprefix.p, kp.data(), sizeof(long long) * (T + 1), hipMemcpyHostToDevice) != hipSuccess ||
                      hipMemcpy(D->sprefix.p, sp.data(), sizeof(long long) * (T + 1), hipMemcpyHostToDevice) != hipSuccess))
    st = GC_ERR_DEVICE;
  if (st != GC_OK) {
    release(D->kprefix);
    release(D->sprefix);
    release(D->qprefix);
    delete D;
    return st;
  }
  ctx->dplans.insert(ctx->dplans.begin(), D);
  while (ctx->dplans.size() > 8) {
    DecPlan* old = ctx->dplans.back();
    ctx->dplans.pop_back();
    (void)hipDeviceSynchronize();
    release(old->kprefix);
    release(old->sprefix);
    release(old->qprefix);
    delete old;
  }
  *out = D;
  return GC_OK;
}

// static_scratch: null, or the device address of the file-scope `scratch` array; the call then takes
// its three work arrays from there instead of the context's workspace and allocates nothing.
gc_status decompress_impl(gc_ctx* ctx, const gc_buf* bufs, int32_t W, const int64_t* k, int32_t T,
                          const int32_t* staleness, bool apply, float c_apply, float* out, int64_t n,
                          void* hip_stream, unsigned char* static_scratch = nullptr) {
  if (!ctx || !bufs || !out || W < 1 || n <= 0) return GC_ERR_INVALID_ARG;
  if (apply && !(c_apply >= 0.0f && c_apply <= 3.0e38f)) return GC_ERR_INVALID_ARG;
  if (W > kMaxWorkers) return GC_ERR_UNSUPPORTED;
  if (reinterpret_cast<uintptr_t>(out) % 4) return GC_ERR_INVALID_ARG;
  const int32_t block = bufs[0].block, ib = bufs[0].index_bits, codec = bufs[0].codec;
  if (block < 1 || (ib != 32 && ib != 64)) return GC_ERR_INVALID_ARG;
  if (codec != GC_CODEC_INT8 && codec != GC_CODEC_SIGN1) return GC_ERR_INVALID_ARG;
  if (ib == 32 && n > (int64_t(1) << 32)) return GC_ERR_INVALID_ARG;
  int64_t ksum = 0;
  if (T > 0) {
    if (!k) return GC_ERR_INVALID_ARG;
    for (int32_t t = 0; t < T; ++t) {
      if (k[t] < 1) return GC_ERR_INVALID_ARG;
      ksum += k[t];
    }
  }
  DecArgs a;
  std::memset(&a, 0, sizeof(a));
  int64_t nrec = 0;  // pairs of all workers
  for (int32_t w = 0; w < W; ++w) {
    const gc_buf& b = bufs[w];
    if (b.n != n || b.block != block || b.index_bits != ib || b.codec != codec || b.k < 0 || b.reserved_ != 0)
      return GC_ERR_INVALID_ARG;
    if (b.k >= (int64_t(1) << 32)) return GC_ERR_UNSUPPORTED;
    if (b.k > 0 && (!b.indices || !b.q || !b.scales)) return GC_ERR_INVALID_ARG;
    if (T > 0 && b.k != ksum) return GC_ERR_INVALID_ARG;
    a.indices[w] = b.indices;
    a.q[w] = b.q;
    a.scales[w] = b.scales;
    a.k[w] = (uint32_t)b.k;
    nrec += b.k;
    a.denom[w] = 1.0f;
    if (staleness) {
      if (staleness[w] < 0 || staleness[w] > (1 << 24)) return GC_ERR_INVALID_ARG;  // 1 + tau exact in fp32
      a.denom[w] = 1.0f + (float)staleness[w];
    }
  }
  GC_HIP(hipSetDevice(ctx->device));
  // the in-place update reads and rewrites scattered words of theta: it needs many wavefronts per
  // compute unit more than it needs large tiles (7B: 5.0 ms with small tiles, 7.0 ms with large ones)
  const int tshift = ctx->opt_dec_large_tile >= 0 ? dec_tile_shift_of(ctx->opt_dec_large_tile != 0)
                     : apply                      ? dec_tile_shift_of(false)
                                                  : dec_tile_shift(nrec, n);
  const int64_t ntiles = (n + (int64_t(1) << tshift) - 1) >> tshift;
  if (ntiles >= (int64_t(1) << 31)) return GC_ERR_UNSUPPORTED;
  const int tb = dec_range_tiles(W, tshift, nrec, n);
  const int64_t nranges = (ntiles + tb - 1) / tb;
  hipStream_t s = (hipStream_t)hip_stream;
  // The one-kernel route reads a tile's pairs straight from the workers' lists and never writes the
  // merged record stream. Its cost per tile grows with the number of workers (every lane looks its
  // pair up among W segments), so it is taken up to 32 workers: measured at n = 5e8, 4 to 32 workers,
  // 3 to 2000 pairs per 4096 floats, it is ahead of the two-kernel route everywhere (1.3B at 0.5 %,
  // 16 workers: 1.6 against 1.8 ms; 7B at 0.1 %: 5.35 against 6.2 ms), and behind it from 48 workers on.
  // Its shape with preparing wavefronts where tiles are thinly filled, the cooperative one where they
  // are crowded or the workers many.
  // The in-place update is faster in one kernel only in a middle band of fillings (at 16 workers,
  // 330 pairs per 4096 floats: 0.96 against 1.21 ms; thin and very crowded tiles: the reverse).
  // The variant that allocates nothing always takes the two-kernel route: that is the route whose
  // scratch arrays it provides.
  const double ppt = (double)nrec * 4096.0 / (double)(n > 0 ? n : 1);  // pairs per 4096 floats of output
  const bool thin = ppt <= 128.0;
  bool fused;
  if (static_scratch) fused = false;
  else if (ctx->opt_dec_fused >= 0) fused = ctx->opt_dec_fused == 1;
  else if (apply) fused = W <= 32 && ppt >= 96.0 && ppt <= 400.0;
  else fused = W <= 32 || (thin && n <= (int64_t(1) << 22));
  const int fused_crowded = ctx->opt_dec_fused_tile >= 0 ? (int)ctx->opt_dec_fused_tile
                                                         : ((ppt >= 128.0 || W > 16 || apply) ? 1 : 0);
  if (fused) {
    // no record stream, no workspace (multi-tensor buffers bring their small prefix tables)
    DecPlan* Df = nullptr;
    if (T > 1) {
      if (static_scratch) return GC_ERR_UNSUPPORTED;
      const gc_status pst = get_dec_plan(ctx, k, T, block, codec, &Df);
      if (pst != GC_OK) return pst;
    }
    Scope sc(static_scratch ? nullptr : ctx, kKDecFused, s);
    launch_dec_fused(a, W, ib, block, codec, staleness ? 1 : 0, n, Df ? (const long long*)Df->kprefix.p : nullptr,
                     Df ? (const long long*)Df->sprefix.p : nullptr, Df ? (const long long*)Df->qprefix.p : nullptr,
                     Df ? T : 1, out, apply ? 1 : 0, c_apply,
                     fused_crowded, s);
    return launch_status();
  }
  const size_t rec_bytes = sizeof(uint2) * (size_t)std::max<int64_t>(nrec, 1);
  const size_t ts_bytes = sizeof(unsigned long long) * (size_t)(ntiles + 1);
  void* rec = nullptr;
  unsigned long long* tile_start = nullptr;
  gc_status st = GC_OK;
  DecPlan* D = nullptr;
  if (static_scratch) {
    // carve the two arrays out of the static array (256-byte pieces); nothing is allocated
    if (T > 1) return GC_ERR_UNSUPPORTED;
    const size_t o_rec = (size_t)round_up((int64_t)ts_bytes, 256);
    if (o_rec + rec_bytes > kStaticScratchBytes) return GC_ERR_UNSUPPORTED;
    tile_start = reinterpret_cast<unsigned long long*>(static_scratch);
    rec = static_scratch + o_rec;
  } else {
    st = ensure(ctx->dec_rec, rec_bytes);
    if (st == GC_OK) st = ensure(ctx->dec_tile_start, ts_bytes);
    if (st != GC_OK) return st;
    if (T > 1) {
      st = get_dec_plan(ctx, k, T, block, codec, &D);
      if (st != GC_OK) return st;
    }
    rec = ctx->dec_rec.p;
    tile_start = (unsigned long long*)ctx->dec_tile_start.p;
  }
  gc_ctx* pc = static_scratch ? nullptr : ctx;  // event pairs are created on demand: not in the static variant
  {
    Scope sc(pc, kKDecPack, s);
    launch_dec_pack(a, W, ib, tb, tshift, block, ntiles, 0, nranges, D ? (const long long*)D->kprefix.p : nullptr,
                    D ? (const long long*)D->sprefix.p : nullptr, D ? (const long long*)D->qprefix.p : nullptr,
                    D ? T : 1, codec, staleness ? 1 : 0, rec, tile_start, s);
  }
  {
    Scope sc(pc, kKDecTiles, s);
    launch_dec_tiles(rec, tile_start, (uint64_t)nrec, tshift, n, 0, ntiles, out, apply ? 1 : 0, c_apply,
                     (unsigned)ctx->opt_apply_dense_min, s);
  }
  return launch_status();
}

gc_status dense_common_check(gc_ctx* ctx, int64_t n, int32_t block, gc_codec codec) {
  if (!ctx || n <= 0 || block < 1) return GC_ERR_INVALID_ARG;
  if (codec != GC_CODEC_INT8 && codec != GC_CODEC_SIGN1) return GC_ERR_INVALID_ARG;
  if (block > kDenseMaxBlock) return GC_ERR_UNSUPPORTED;
  if ((n + block - 1) / block >= (int64_t(1) << 31) - (int64_t(1) << 20)) return GC_ERR_UNSUPPORTED;  // padded grid
  return GC_OK;
}

gc_status dense_sum_impl(gc_ctx* ctx, const void* const* q, const float* const* scales, int32_t W, int32_t block,
                         gc_codec codec, const int32_t* staleness, bool apply, float c_apply, float* out,
                         int64_t n, void* hip_stream) {
  gc_status st = dense_common_check(ctx, n, block, codec);
  if (st != GC_OK) return st;
  if (!q || !scales || !out || W < 1) return GC_ERR_INVALID_ARG;
  if (W > kMaxWorkers) return GC_ERR_UNSUPPORTED;
  if (apply && !(c_apply >= 0.0f && c_apply <= 3.0e38f)) return GC_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(out) % 4) return GC_ERR_INVALID_ARG;
  if ((n + 1023) / 1024 >= (int64_t(1) << 31)) return GC_ERR_UNSUPPORTED;
  DenseDecArgs a;
  std::memset(&a, 0, sizeof(a));
  for (int32_t w = 0; w < W; ++w) {
    if (!q[w] || !scales[w] || (reinterpret_cast<uintptr_t>(scales[w]) % 4)) return GC_ERR_INVALID_ARG;
    a.q[w] = static_cast<const int8_t*>(q[w]);
    a.scales[w] = scales[w];
    a.denom[w] = 1.0f;
    if (staleness) {
      if (staleness[w] < 0 || staleness[w] > (1 << 24)) return GC_ERR_INVALID_ARG;
      a.denom[w] = 1.0f + (float)staleness[w];
    }
  }
  GC_HIP(hipSetDevice(ctx->device));
  hipStream_t s = (hipStream_t)hip_stream;
  {
    Scope sc(ctx, kKDenseSum, s);
    launch_dense_sum(a, W, block, n, (int)codec, out, staleness ? 1 : 0, apply ? 1 : 0, c_apply, s);
  }
  return launch_status();
}

const char* const kKernelNames[kKNum] = {"k_sample", "k_sample_thresh", "k_main", "k_group_sums", "k_group_scan",
                                         "k_route", "k_gather", "k_hist", "k_select_scan", "k_count",
                                         "k_chunk_sums", "k_chunk_scan", "k_emit", "k_quant", "k_finish", "k_dec_pack", "k_dec_tiles", "k_dec_fused",
                                         "k_dense", "k_dense_sum", "k_rows_gather", "k_rows_finish", "k_rows_remap"};

}  // namespace

extern "C" {

gc_status gc_create(gc_ctx** out, int device) {
  if (!out) return GC_ERR_INVALID_ARG;
  *out = nullptr;
  int count = 0;
  if (hipGetDeviceCount(&count) != hipSuccess) {
    (void)hipGetLastError();
    return GC_ERR_DEVICE;
  }
  if (device < 0 || device >= count) return GC_ERR_INVALID_ARG;
  GC_HIP(hipSetDevice(device));
  if (device < kMaxDevices) {  // this device's copy of the static scratch array: looked up once
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[device]) {
      void* p = nullptr;
      if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
        (void)hipGetLastError();
        return GC_ERR_DEVICE;
      }
      g_scratch_ptr[device] = p;
    }
  }
  gc_ctx* c = new (std::nothrow) gc_ctx();
  if (!c) return GC_ERR_WORKSPACE;
  c->device = device;
  gc_status st = ensure(c->flags, sizeof(uint32_t) * 4);
  if (st == GC_OK && hipMemset(c->flags.p, 0, sizeof(uint32_t) * 4) != hipSuccess) st = GC_ERR_DEVICE;
  if (st == GC_OK && hipHostMalloc((void**)&c->host_flags, sizeof(uint32_t) * 4, hipHostMallocDefault) != hipSuccess)
    st = GC_ERR_WORKSPACE;
  if (st != GC_OK) {
    (void)hipGetLastError();
    release(c->flags);
    if (c->host_flags) (void)hipHostFree(c->host_flags);
    delete c;
    return st;
  }
  *out = c;
  return GC_OK;
}

gc_status gc_reserve(gc_ctx* ctx, int64_t max_n, int64_t max_k, int32_t max_tensors, int32_t max_W) {
  if (!ctx || max_n < 1 || max_k < 1 || max_k > max_n || max_tensors < 1 || max_W < 0 || max_W > kMaxWorkers)
    return GC_ERR_INVALID_ARG;
  if (max_k >= (int64_t(1) << 32)) return GC_ERR_UNSUPPORTED;
  GC_HIP(hipSetDevice(ctx->device));
  // Every array grows with n, k and the tensor count; the candidate slots also grow with the
  // density k / n. The bound is the plan of one tensor of max_n elements keeping max_k (block 1:
  // the most scales), widened by what max_tensors tensors add at their boundaries.
  const int64_t offsets[2] = {0, max_n};
  Plan* P = build_plan(offsets, &max_k, 1, 1, GC_CODEC_INT8);
  if (!P) return GC_ERR_WORKSPACE;
  Need nd = need_of(P);
  const size_t T = (size_t)max_tensors;
  const int32_t slot_stride = std::max(P->slot_stride, kSlotLine);
  delete P;
  nd.T = T;
  nd.ngroups += 2 * T;
  nd.max_chunks += 2 * T;
  nd.sampled = true;
  nd.slot_records = nd.ngroups * (size_t)slot_stride;
  nd.cand = (size_t)std::min<int64_t>(max_n, 8 * max_k) + 4100 * T;
  gc_status st = ensure_workspace(ctx, nd);
  // the row-sparse step and the aggregates
  if (st == GC_OK) st = ensure(ctx->rows_e, sizeof(float) * (size_t)max_n);
  if (st == GC_OK) st = ensure(ctx->rows_idx, sizeof(uint32_t) * (size_t)max_k);
  if (max_W > 0) {
    const size_t pairs = (size_t)max_W * (size_t)max_k;
    if (st == GC_OK) st = ensure(ctx->rows_cidx, sizeof(uint32_t) * pairs);
    if (st == GC_OK) st = ensure(ctx->dec_rec, sizeof(uint2) * pairs);
    if (st == GC_OK) st = ensure(ctx->dec_tile_start, sizeof(unsigned long long) * (size_t)((max_n >> kDecMinTileShift) + 2));
  }
  return st;
}

gc_status gc_destroy(gc_ctx* c) {
  if (!c) return GC_ERR_INVALID_ARG;
  (void)hipSetDevice(c->device);
  (void)hipDeviceSynchronize();
  for (Plan* P : c->plans) { release(P->td_dev); release(P->recs_dev); delete P; }
  delete c->single;
  for (DecPlan* D : c->dplans) { release(D->kprefix); release(D->sprefix); release(D->qprefix); delete D; }
  DevBuf* all[] = {&c->ts, &c->shist, &c->hist, &c->grp_cnt, &c->grp_part, &c->grp_off, &c->tg_base,
                   &c->slots, &c->cand_val, &c->cand_idx, &c->ch_gt, &c->ch_eq,
                   &c->ch_part_gt, &c->ch_part_eq, &c->ch_goff, &c->ch_eoff, &c->tb_g, &c->tb_e,
                   &c->totals, &c->kept_val, &c->flags, &c->dec_rec, &c->dec_tile_start, &c->rows_e, &c->rows_idx, &c->rows_cidx};
  for (DevBuf* b : all) release(*b);
  if (c->host_flags) (void)hipHostFree(c->host_flags);
  if (c->host_ts) (void)hipHostFree(c->host_ts);
  for (auto& e : c->ev_used) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
  for (auto& e : c->ev_free) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
  delete c;
  return GC_OK;
}

int64_t gc_k_from_density(int64_t n, double density) {
  if (n <= 0) return 0;
  const double kd = std::ceil((double)n * density);
  if (!(kd >= 1.0)) return 1;
  if (kd >= (double)n) return n;
  return (int64_t)kd;
}

int64_t gc_num_code_bytes(int64_t k, int32_t block, gc_codec codec) {
  if (codec != GC_CODEC_INT8 && codec != GC_CODEC_SIGN1) return 0;
  return code_bytes(k, block, (int32_t)codec);
}

int64_t gc_num_scales(int64_t k, int32_t block) {
  if (k <= 0 || block < 1) return 0;
  return (k + block - 1) / block;
}

gc_status gc_compress(gc_ctx* ctx, const void* grad, gc_dtype dtype, float* residual, int64_t n, int64_t k,
                      int32_t block, const gc_buf* out, void* hip_stream) {
  if (n <= 0) return GC_ERR_INVALID_ARG;
  const int64_t offsets[2] = {0, n};
  return compress_impl(ctx, grad, dtype, residual, offsets, &k, 1, block, out, hip_stream);
}

gc_status gc_compress_multi(gc_ctx* ctx, const void* grad, gc_dtype dtype, float* residual,
                            const int64_t* offsets, const int64_t* k, int32_t T, int32_t block,
                            const gc_buf* out, void* hip_stream) {
  return compress_impl(ctx, grad, dtype, residual, offsets, k, T, block, out, hip_stream);
}

gc_status gc_decompress_sum(gc_ctx* ctx, const gc_buf* bufs, int32_t W, float* out, int64_t n,
                            void* hip_stream) {
  return decompress_impl(ctx, bufs, W, nullptr, 0, nullptr, false, 0.0f, out, n, hip_stream);
}

gc_status gc_decompress_sum_static(gc_ctx* ctx, const gc_buf* bufs, int32_t W, float* out, int64_t n,
                                   void* hip_stream) {
  if (!ctx) return GC_ERR_INVALID_ARG;
  if (ctx->device < 0 || ctx->device >= kMaxDevices) return GC_ERR_UNSUPPORTED;
  unsigned char* sp = nullptr;
  {
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    sp = static_cast<unsigned char*>(g_scratch_ptr[ctx->device]);  // set by gc_create on this device
  }
  if (!sp) return GC_ERR_DEVICE;
  return decompress_impl(ctx, bufs, W, nullptr, 0, nullptr, false, 0.0f, out, n, hip_stream, sp);
}

gc_status gc_decompress_sum_weighted(gc_ctx* ctx, const gc_buf* bufs, int32_t W, const int64_t* k, int32_t T,
                                     const int32_t* staleness, float* out, int64_t n, void* hip_stream) {
  if (!staleness || T < 0) return GC_ERR_INVALID_ARG;
  return decompress_impl(ctx, bufs, W, k, T, staleness, false, 0.0f, out, n, hip_stream);
}

gc_status gc_decompress_apply(gc_ctx* ctx, const gc_buf* bufs, int32_t W, const int64_t* k, int32_t T,
                              const int32_t* staleness, float* theta, float step, int64_t n,
                              void* hip_stream) {
  if (T < 0) return GC_ERR_INVALID_ARG;
  return decompress_impl(ctx, bufs, W, k, T, staleness, true, step, theta, n, hip_stream);
}

gc_status gc_decompress_sum_multi(gc_ctx* ctx, const gc_buf* bufs, int32_t W, const int64_t* k, int32_t T,
                                  float* out, int64_t n, void* hip_stream) {
  if (T < 1) return GC_ERR_INVALID_ARG;
  return decompress_impl(ctx, bufs, W, k, T, nullptr, false, 0.0f, out, n, hip_stream);
}

gc_status gc_compress_rows(gc_ctx* ctx, const void* vals, gc_dtype dtype, float* residual_table,
                           const int64_t* rows, int64_t U, int64_t D, int64_t R, int64_t k, int32_t block,
                           const gc_buf* out, void* hip_stream) {
  if (!ctx || !vals || !residual_table || !rows || !out) return GC_ERR_INVALID_ARG;
  if (U < 1 || D < 1 || R < 1 || U > R || block < 1) return GC_ERR_INVALID_ARG;
  int64_t m = 0, table = 0;  // compact length (its positions must fit 32 bits) and table length
  if (__builtin_mul_overflow(U, D, &m) || m >= (int64_t(1) << 32)) return GC_ERR_UNSUPPORTED;
  if (__builtin_mul_overflow(R, D, &table) || table >= (int64_t(1) << 62)) return GC_ERR_UNSUPPORTED;
  if (k < 1 || k > m) return GC_ERR_INVALID_ARG;
  if (out->n != table || out->k != k || out->block != block) return GC_ERR_INVALID_ARG;
  if (out->index_bits != 32 && out->index_bits != 64) return GC_ERR_INVALID_ARG;
  if (out->index_bits == 32 && table > (int64_t(1) << 32)) return GC_ERR_INVALID_ARG;
  if (!out->indices || !out->q || !out->scales) return GC_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(rows) % 8) || (reinterpret_cast<uintptr_t>(residual_table) % 4) ||
      (reinterpret_cast<uintptr_t>(out->indices) % (out->index_bits / 8)))
    return GC_ERR_INVALID_ARG;
  GC_HIP(hipSetDevice(ctx->device));
  gc_status st = ensure(ctx->rows_e, sizeof(float) * (size_t)m);
  if (st == GC_OK) st = ensure(ctx->rows_idx, sizeof(uint32_t) * (size_t)k);
  if (st != GC_OK) return st;
  // the flat step on the compact tensor; argument errors surface here, before anything is written
  gc_buf tmp = *out;
  tmp.indices = ctx->rows_idx.p;
  tmp.n = m;
  tmp.index_bits = 32;
  hipStream_t s = (hipStream_t)hip_stream;
  float* ec = (float*)ctx->rows_e.p;
  const long long* rws = reinterpret_cast<const long long*>(rows);
  {
    // the gather only reads caller memory and writes scratch, so running it before the flat
    // step's own argument check writes nothing the caller can see
    Scope sc(ctx, kKRowsGather, s);
    launch_rows_gather(residual_table, rws, U, D, R, ec, (uint32_t*)ctx->flags.p, s);
  }
  const int64_t offsets[2] = {0, m};
  st = compress_impl(ctx, vals, dtype, ec, offsets, &k, 1, block, &tmp, hip_stream);
  if (st != GC_OK) return st;
  {
    Scope sc(ctx, kKRowsFinish, s);
    launch_rows_finish(residual_table, rws, U, D, R, ec, (const uint32_t*)ctx->rows_idx.p, k, out->indices,
                       out->index_bits, s);
  }
  return launch_status();
}

gc_status gc_decompress_sum_rows(gc_ctx* ctx, const gc_buf* bufs, int32_t W, const int64_t* urows, int64_t Ru,
                                 int64_t D, const int32_t* staleness, float* out, void* hip_stream) {
  if (!ctx || !bufs || !urows || !out || W < 1 || Ru < 1 || D < 1) return GC_ERR_INVALID_ARG;
  if (W > kMaxWorkers) return GC_ERR_UNSUPPORTED;
  int64_t m = 0;  // length of the compact aggregate: its positions must fit 32 bits
  if (__builtin_mul_overflow(Ru, D, &m) || m >= (int64_t(1) << 32)) return GC_ERR_UNSUPPORTED;
  if (reinterpret_cast<uintptr_t>(urows) % 8) return GC_ERR_INVALID_ARG;
  int64_t ktotal = 0;
  for (int32_t w = 0; w < W; ++w) {
    const gc_buf& b = bufs[w];
    if (b.k < 0 || b.k >= (int64_t(1) << 32) || (b.index_bits != 32 && b.index_bits != 64) || b.reserved_ != 0)
      return GC_ERR_INVALID_ARG;
    if (b.k > 0 && (!b.indices || !b.q || !b.scales)) return GC_ERR_INVALID_ARG;
    ktotal += b.k;
  }
  GC_HIP(hipSetDevice(ctx->device));
  gc_status st = ensure(ctx->rows_cidx, sizeof(uint32_t) * (size_t)std::max<int64_t>(ktotal, 1));
  if (st != GC_OK) return st;
  hipStream_t s = (hipStream_t)hip_stream;
  std::vector<gc_buf> tmp(bufs, bufs + W);
  uint32_t* cidx = (uint32_t*)ctx->rows_cidx.p;
  if (ktotal >= (int64_t(1) << 32)) return GC_ERR_UNSUPPORTED;
  RowsRemapArgs ra;
  std::memset(&ra, 0, sizeof(ra));
  int64_t at = 0;
  for (int32_t w = 0; w < W; ++w) {
    ra.idx[w] = bufs[w].indices;
    ra.k[w] = (uint32_t)bufs[w].k;
    ra.at[w] = (uint32_t)at;
    ra.bits[w] = (uint8_t)bufs[w].index_bits;
    tmp[w].indices = cidx + at;
    tmp[w].index_bits = 32;
    tmp[w].n = m;
    at += bufs[w].k;
  }
  {
    Scope sc(ctx, kKRowsRemap, s);
    launch_rows_remap(ra, W, reinterpret_cast<const long long*>(urows), Ru, D, cidx, (uint32_t*)ctx->flags.p, s);
  }
  return decompress_impl(ctx, tmp.data(), W, nullptr, 0, staleness, false, 0.0f, out, m, hip_stream);
}

gc_status gc_compress_dense(gc_ctx* ctx, const void* grad, gc_dtype dtype, float* residual, int64_t n,
                            int32_t block, gc_codec codec, void* q, float* scales, void* hip_stream) {
  gc_status st = dense_common_check(ctx, n, block, codec);
  if (st != GC_OK) return st;
  if (!grad || !residual || !q || !scales) return GC_ERR_INVALID_ARG;
  if (dtype != GC_F32 && dtype != GC_BF16) return GC_ERR_INVALID_ARG;
  const size_t gsz = dtype == GC_F32 ? 4 : 2;
  if ((reinterpret_cast<uintptr_t>(grad) % gsz) || (reinterpret_cast<uintptr_t>(residual) % 4) ||
      (reinterpret_cast<uintptr_t>(scales) % 4))
    return GC_ERR_INVALID_ARG;
  GC_HIP(hipSetDevice(ctx->device));
  hipStream_t s = (hipStream_t)hip_stream;
  {
    Scope sc(ctx, kKDense, s);
    launch_dense(grad, (int)dtype, residual, n, block, (int)codec, q, scales, nullptr, 0, (uint32_t*)ctx->flags.p,
                 (int)ctx->opt_dense_wave_block, (int)ctx->opt_dense_lds_pad, s);
  }
  ctx->last_plan = nullptr;
  ctx->last_dense_tensors = 1;
  return launch_status();
}

gc_status gc_decompress_sum_dense(gc_ctx* ctx, const void* const* q, const float* const* scales, int32_t W,
                                  int32_t block, gc_codec codec, const int32_t* staleness, float* out,
                                  int64_t n, void* hip_stream) {
  return dense_sum_impl(ctx, q, scales, W, block, codec, staleness, false, 0.0f, out, n, hip_stream);
}

gc_status gc_decompress_apply_dense(gc_ctx* ctx, const void* const* q, const float* const* scales, int32_t W,
                                    int32_t block, gc_codec codec, const int32_t* staleness, float* theta,
                                    float step, int64_t n, void* hip_stream) {
  return dense_sum_impl(ctx, q, scales, W, block, codec, staleness, true, step, theta, n, hip_stream);
}

gc_status gc_sync_status(gc_ctx* ctx, void* hip_stream) {
  if (!ctx) return GC_ERR_INVALID_ARG;
  GC_HIP(hipSetDevice(ctx->device));
  hipStream_t s = (hipStream_t)hip_stream;
  GC_HIP(hipMemcpyAsync(ctx->host_flags, ctx->flags.p, sizeof(uint32_t) * 4, hipMemcpyDeviceToHost, s));
  if (ctx->last_plan)
    GC_HIP(hipMemcpyAsync(ctx->host_ts, ctx->ts.p, sizeof(TensorState) * ctx->last_plan->td.size(),
                          hipMemcpyDeviceToHost, s));
  GC_HIP(hipStreamSynchronize(s));
  const bool bad_rows = ctx->host_flags[1] != 0u;
  const bool bad = ctx->host_flags[0] != 0u || bad_rows;
  if (bad) {
    GC_HIP(hipMemsetAsync(ctx->flags.p, 0, sizeof(uint32_t) * 4, s));
    GC_HIP(hipStreamSynchronize(s));
  }
  if (bad_rows) return GC_ERR_INVALID_ARG;  // a row id out of range or out of order (gc_compress_rows)
  return bad ? GC_ERR_NONFINITE : GC_OK;
}

gc_status gc_last_stats(gc_ctx* ctx, gc_stats* stats) {
  if (!ctx || !stats) return GC_ERR_INVALID_ARG;
  std::memset(stats, 0, sizeof(*stats));
  const Plan* P = ctx->last_plan;
  if (!P) {
    stats->tensors = ctx->last_dense_tensors;
    return GC_OK;
  }
  stats->tensors = (int64_t)P->td.size();
  for (size_t t = 0; t < P->td.size(); ++t) {
    if (P->td[t].mode != kSampled) continue;
    stats->tensors_sampled++;
    const TensorState& st = ctx->host_ts[t];
    stats->candidates += (int64_t)st.cand_total;
    if (!st.use_cand) stats->tensors_fallback++;
  }
  return GC_OK;
}

gc_status gc_profile_enable(gc_ctx* ctx, int32_t on) {
  if (!ctx) return GC_ERR_INVALID_ARG;
  GC_HIP(hipSetDevice(ctx->device));
  GC_HIP(hipDeviceSynchronize());
  for (auto& e : ctx->ev_used) ctx->ev_free.push_back(e);
  ctx->ev_used.clear();
  ctx->prof = (on == 2) ? 2 : (on != 0 ? 1 : 0);
  return GC_OK;
}

gc_status gc_set_option(gc_ctx* ctx, const char* name, int64_t value) {
  if (!ctx || !name) return GC_ERR_INVALID_ARG;
  if (std::strcmp(name, "main_lds_pad") == 0) {
    if (value < 0 || value > 65536) return GC_ERR_INVALID_ARG;
    ctx->opt_main_lds_pad = value;
    return GC_OK;
  }
  if (std::strcmp(name, "dense_wave_block") == 0) {
    if (value < 0 || value > 2048) return GC_ERR_INVALID_ARG;
    ctx->opt_dense_wave_block = value;
    return GC_OK;
  }
  if (std::strcmp(name, "dec_large_tile") == 0) {
    if (value < -1 || value > 1) return GC_ERR_INVALID_ARG;
    ctx->opt_dec_large_tile = value;
    return GC_OK;
  }
  if (std::strcmp(name, "dec_fused_tile") == 0) {
    if (value < -1 || value > 1) return GC_ERR_INVALID_ARG;
    ctx->opt_dec_fused_tile = value;
    return GC_OK;
  }
  if (std::strcmp(name, "dec_fused") == 0) {
    if (value < -1 || value > 1) return GC_ERR_INVALID_ARG;
    ctx->opt_dec_fused = value;
    return GC_OK;
  }
  if (std::strcmp(name, "apply_dense_min") == 0) {
    if (value < 1 || value > (int64_t(1) << 30)) return GC_ERR_INVALID_ARG;
    ctx->opt_apply_dense_min = value;
    return GC_OK;
  }
  if (std::strcmp(name, "dense_lds_pad") == 0) {
    if (value < -1 || value > 65536) return GC_ERR_INVALID_ARG;
    ctx->opt_dense_lds_pad = value;
    return GC_OK;
  }
  return GC_ERR_INVALID_ARG;
}

int32_t gc_profile_num_kernels(void) { return kKNum; }

const char* gc_profile_kernel_name(int32_t id) { return (id >= 0 && id < kKNum) ? kKernelNames[id] : ""; }

gc_status gc_profile_read(gc_ctx* ctx, int32_t id, double* total_ms, int64_t* launches) {
  if (!ctx || !total_ms || !launches || id < 0 || id >= kKNum) return GC_ERR_INVALID_ARG;
  GC_HIP(hipSetDevice(ctx->device));
  double tot = 0.0;
  int64_t cnt = 0;
  for (auto& e : ctx->ev_used) {
    if (e.id != id) continue;
    GC_HIP(hipEventSynchronize(e.b));
    float ms = 0.0f;
    GC_HIP(hipEventElapsedTime(&ms, e.a, e.b));
    tot += ms;
    ++cnt;
  }
  *total_ms = tot;
  *launches = cnt;
  return GC_OK;
}

const char* gc_status_string(gc_status s) {
  switch (s) {
    case GC_OK: return "ok";
    case GC_ERR_INVALID_ARG: return "invalid argument";
    case GC_ERR_UNSUPPORTED: return "unsupported size";
    case GC_ERR_WORKSPACE: return "workspace allocation failed";
    case GC_ERR_NONFINITE: return "non-finite value among the kept entries";
    case GC_ERR_DEVICE: return "HIP runtime error";
  }
  return "unknown status";
}

}  // extern "C"
