/* gradcomp — error-feedback top-k gradient compression with per-block int8
 * quantization, and the matching decompress-and-sum, for one MI355X (gfx950).
 *
 * C ABI. Every data pointer is DEVICE memory owned by the caller unless a
 * comment says "host". The library allocates only its own scratch workspace
 * (inside gc_ctx); it never frees or resizes caller memory. All work is queued
 * on the HIP stream the caller passes (a hipStream_t cast to void*; NULL is the
 * default stream) and the calls return without waiting for it. Argument errors
 * are returned at once and nothing is written. Conditions that only the device
 * can see (a non-finite value among the kept entries) are reported by
 * gc_sync_status().
 *
 * One gc_ctx serves one stream at a time: two calls that use the same ctx from
 * different streams without ordering between them race on its workspace.
 *
 * The method (paper Sec. III.B): each worker sends only the k entries of
 * largest magnitude of its accumulated gradient and keeps the rest as a
 * residual that re-enters the next step, Eq. (11): r_{t+1} = r_t + g - ghat.
 * The receiver forms the aggregate of the workers' (compressed) gradients,
 * Eq. (8); here that aggregate is returned as the plain sum, the 1/P factor is
 * left to the caller.
 */
#ifndef GRADCOMP_H
#define GRADCOMP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GC_OK = 0,
  GC_ERR_INVALID_ARG = 1, /* null pointer, size out of range, mismatched buffers */
  GC_ERR_UNSUPPORTED = 2, /* valid request this build cannot serve (e.g. W too large) */
  GC_ERR_WORKSPACE = 3,   /* scratch allocation failed */
  GC_ERR_NONFINITE = 4,   /* Inf/NaN among the kept entries; outputs unspecified */
  GC_ERR_DEVICE = 5       /* a HIP runtime call failed */
} gc_status;

typedef enum { GC_F32 = 0, GC_BF16 = 1 } gc_dtype;

/* How the kept values are coded.
 * GC_CODEC_INT8:  one int8 per pair and one fp32 scale per block, s = amax / 127,
 *                 q = rint(v / s); decodes to fl32(q * s).
 * GC_CODEC_SIGN1: the paper's 1-bit quantizer (Sec. III.B, Eq. 10): one sign bit per pair (set when
 *                 v >= 0) and one fp32 scale per block, the block's mean magnitude ||v||_1 / len
 *                 (l1 sum in fp64 over a balanced binary tree, then one division, one rounding);
 *                 decodes to +s or -s. Bits are packed 8 per byte, least significant first, every
 *                 block starting a new byte. Needs block <= 8192. */
typedef enum { GC_CODEC_INT8 = 0, GC_CODEC_SIGN1 = 1 } gc_codec;

typedef struct gc_ctx gc_ctx; /* opaque; owns scratch workspace on one device */

/* A compressed gradient: k (index, code) pairs in ascending index order plus one
 * fp32 scale per block of `block` consecutive pairs (the last block may be
 * short). Entry j decodes to (float)q[j] * scales[j / block], rounded to fp32.
 * For a multi-tensor buffer the pairs of all tensors are concatenated in tensor
 * order, indices are positions in the flat buffer, and blocks restart at every
 * tensor boundary (scales are concatenated the same way). */
typedef struct {
  void* indices;      /* k entries; uint32_t if index_bits == 32, uint64_t if 64 */
  int8_t* q;          /* gc_num_code_bytes(k, block, codec) bytes: k codes in [-127, 127], or sign bits */
  float* scales;      /* gc_num_scales(k, block) entries (multi: sum over tensors) */
  int64_t n;          /* length of the dense vector the indices point into */
  int64_t k;          /* number of pairs */
  int32_t block;      /* pairs per scale */
  int32_t index_bits; /* 32 or 64; must be 64 when n > 2^32 */
  int32_t codec;      /* gc_codec of the values */
  int32_t reserved_;  /* must be 0 */
} gc_buf;

/* Counters of the last compress call, valid after gc_sync_status(). */
typedef struct {
  int64_t tensors;          /* tensors in the call */
  int64_t tensors_sampled;  /* tensors whose candidates were gathered in the streaming pass */
  int64_t tensors_fallback; /* of those, how many had to be re-selected from the dense residual */
  int64_t candidates;       /* candidate entries gathered by the streaming pass */
} gc_stats;

/* Create / destroy a context on HIP device `device`. Workspace grows on the
 * first call that needs more of it (that call waits for the device, frees and allocates);
 * gc_reserve sizes it ahead of time. */
gc_status gc_create(gc_ctx** ctx, int device);
gc_status gc_destroy(gc_ctx* ctx);

/* Size the workspace once, so that later calls neither allocate nor wait: after it, every
 * single-tensor call (gc_compress, gc_compress_rows, the aggregates over up to max_W buffers of up
 * to max_k pairs each, gc_decompress_sum_rows) with n (for rows: U * D) <= max_n and k <= max_k only
 * queues kernels on the caller's stream, whatever its exact shape - such calls may sit inside a
 * stream capture and their shape may change from call to call. Multi-tensor calls
 * (gc_compress_multi, gc_decompress_sum_multi) with up to max_tensors tensors, max_n elements and
 * max_k pairs in total, and no tensor denser than max_k / max_n, find the workspace large enough too,
 * but still upload a small per-shape plan the first time a shape (offsets, k, block, code) is seen
 * (eight shapes are remembered). Waits for the device once if anything has to grow.
 * 1 <= max_k <= max_n, max_tensors >= 1, 0 <= max_W <= 64 (0: no aggregate workspace). */
gc_status gc_reserve(gc_ctx* ctx, int64_t max_n, int64_t max_k, int32_t max_tensors, int32_t max_W);

/* k = clamp(ceil(n * density), 1, n), n * density evaluated in IEEE double.
 * Pure host function. The paper names no k; this is the rule the workloads use. */
int64_t gc_k_from_density(int64_t n, double density);

/* ceil(k / block): number of scales for k pairs. Pure host function. */
int64_t gc_num_scales(int64_t k, int32_t block);

/* Bytes of `q` for k pairs of ONE tensor (multi-tensor buffers: the sum over tensors): k for
 * GC_CODEC_INT8; for GC_CODEC_SIGN1 every full block takes ceil(block / 8) bytes and the last,
 * shorter block ceil(len / 8). Pure host function; 0 on invalid arguments. */
int64_t gc_num_code_bytes(int64_t k, int32_t block, gc_codec codec);

/* One error-feedback step of one worker on one flat tensor (Sec. III.B, Eq. 11):
 *   acc = residual + grad            (one fp32 add per entry; bf16 grad is widened exactly)
 *   kept = the k entries of largest |acc| (31-bit magnitude pattern; ties to the lower index)
 *   out  = kept indices ascending, int8 codes q = rint(acc / s) with s = amax/127 per block
 *          of `block` consecutive kept entries (a zero or subnormal s sends the block as zeros)
 *   residual = acc - fl32(q * s) at kept entries, acc elsewhere          (updated in place)
 * grad: n entries of `dtype`, read only. residual: n fp32. 1 <= k <= n, block >= 1,
 * k < 2^32. out->indices/q/scales must hold k / gc_num_code_bytes(k, block, codec) /
 * gc_num_scales(k, block) entries; out->n, out->k, out->block must equal n, k, block.
 * out->codec chooses the value code (the description above is GC_CODEC_INT8; with GC_CODEC_SIGN1
 * the residual at a kept entry is acc -/+ s).
 * Cost: one pass over grad and residual (12 bytes per element) plus work on about 1.2 k candidate
 * entries. The result never depends on the data, the time can: when more than 8 k + 4096 entries tie
 * with or exceed the candidate threshold (fewer non-zeros than k, all-equal values, values on a
 * coarse grid) or k > n / 8, the k-th magnitude is selected from the whole residual: one more pass
 * when a single huge tie holds the threshold (1.6 to 1.9 times the time of the streaming pass in
 * all), four more passes otherwise (3 to 4 times); gc_last_stats() counts such tensors. */
gc_status gc_compress(gc_ctx* ctx, const void* grad, gc_dtype dtype, float* residual, int64_t n,
                      int64_t k, int32_t block, const gc_buf* out, void* hip_stream);

/* The same step for T tensors stored back to back in one flat buffer, each with
 * its own top-k and its own quantization blocks, in one set of launches.
 * offsets: T+1 host entries, offsets[0] = 0, strictly increasing; tensor t is
 * [offsets[t], offsets[t+1]). k: T host entries, 1 <= k[t] <= n_t. `out` is one
 * flat buffer with out->n = offsets[T], out->k = sum k[t] and
 * sum gc_num_scales(k[t], block) scales. */
gc_status gc_compress_multi(gc_ctx* ctx, const void* grad, gc_dtype dtype, float* residual,
                            const int64_t* offsets, const int64_t* k, int32_t T, int32_t block,
                            const gc_buf* out, void* hip_stream);

/* Aggregate of W workers' compressed gradients as a dense vector (Eq. 8 without
 * the 1/P): out[i] = sum over w = 0..W-1, in that order and in fp32, of the
 * decoded value of worker w at i (0 where w sent nothing). `out` (n fp32) is
 * fully overwritten. bufs: W host structs; all must have n == `n` and the same
 * block, index_bits and codec; indices must be ascending and unique within a buffer
 * (as gc_compress writes them). 1 <= W <= 64. */
gc_status gc_decompress_sum(gc_ctx* ctx, const gc_buf* bufs, int32_t W, float* out, int64_t n,
                            void* hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): gc_decompress_sum for single-tensor buffers, with the
 * same result bit for bit, that allocates nothing - no hipMalloc, no hipFree, no workspace growth,
 * no events. It always runs the two-kernel route of the aggregate, whatever gc_decompress_sum would
 * choose; that route's work arrays (the merged record stream, tile starts) live in one static device array
 * of GC_STATIC_SCRATCH_BYTES that every device the library runs on holds until the process ends. A
 * call whose arrays would not fit returns GC_ERR_UNSUPPORTED and writes nothing:
 *   8 * (ceil(n / 4096) + 1) + 8 * (sum of the buffers' k) + 256
 * bytes is an upper bound on what a call takes (e.g. n = 2^30 with 3,900,000 pairs in all).
 * All calls on one device share that array, and it keeps the last call's contents (every call
 * rewrites all it reads, nothing has to start at zero): calls that overlap in time on one device,
 * from any context or stream, race. The context only names the device. */
#define GC_STATIC_SCRATCH_BYTES (32 * 1024 * 1024)
gc_status gc_decompress_sum_static(gc_ctx* ctx, const gc_buf* bufs, int32_t W, float* out, int64_t n,
                                   void* hip_stream);

/* The same for buffers written by gc_compress_multi: k holds the T per-tensor
 * counts (host; identical for every worker), so that scales are looked up per
 * tensor. */
gc_status gc_decompress_sum_multi(gc_ctx* ctx, const gc_buf* bufs, int32_t W, const int64_t* k,
                                  int32_t T, float* out, int64_t n, void* hip_stream);

/* Staleness-damped aggregate (Sec. III.B, Eq. 12: a gradient that is tau steps late enters the
 * update divided by 1 + tau): out[i] = sum over w, in worker order and in fp32, of
 * fl32(d_w[i] / (1 + staleness[w])), d_w the decoded value of worker w. staleness: W host
 * entries in [0, 2^24]. With every staleness 0 the result equals gc_decompress_sum bit for bit.
 * k/T as in gc_decompress_sum_multi, or k = NULL, T = 0 for single-tensor buffers. */
gc_status gc_decompress_sum_weighted(gc_ctx* ctx, const gc_buf* bufs, int32_t W, const int64_t* k, int32_t T,
                                     const int32_t* staleness, float* out, int64_t n, void* hip_stream);

/* Fused aggregate-and-apply (Eq. 8 and Eq. 9): theta[i] <- theta[i] - fl32(step * S[i]), where
 * S is the aggregate gc_decompress_sum (staleness == NULL) or gc_decompress_sum_weighted would
 * write, and `step` stands for eta / P (0 <= step, finite). Only positions named by some
 * buffer are read and written: where S[i] is +0 the update leaves theta[i] unchanged, so the
 * dense aggregate is never materialised. theta: n fp32, updated in place. */
gc_status gc_decompress_apply(gc_ctx* ctx, const gc_buf* bufs, int32_t W, const int64_t* k, int32_t T,
                              const int32_t* staleness, float* theta, float step, int64_t n,
                              void* hip_stream);

/* One error-feedback step on a ROW-SPARSE gradient (the gradient of an embedding table of R rows x D
 * columns of which this step touched U rows; Sec. III.B, Eq. 11, with the residual kept in the shape
 * of the table). Only the touched rows take part: acc = vals + residual_table[rows], the k largest
 * |acc| among those U * D entries are kept and coded as in gc_compress, and residual_table[rows] is
 * rewritten; every other row of the residual is neither read nor written. The paper does not treat
 * sparse gradients; this is the reading under which "density applied to the touched rows" means
 * something, and it makes the step equal to gc_compress on the compacted (U x D) tensor.
 * vals: U * D entries of `dtype`, row-major, in the order of `rows`. rows: U int64 row ids in DEVICE
 * memory, ascending, unique, each in [0, R). residual_table: R * D fp32. 1 <= k <= U * D < 2^32.
 * out->indices receive positions in the table, row * D + column (ascending); out->n must be R * D,
 * out->index_bits 64 when R * D > 2^32; q and scales as for gc_compress with k pairs. The buffers can
 * be passed to gc_decompress_sum with n = R * D. A row id that is out of range or out of order is
 * never dereferenced; the call is then reported by gc_sync_status() as GC_ERR_INVALID_ARG and its
 * outputs are unspecified. */
gc_status gc_compress_rows(gc_ctx* ctx, const void* vals, gc_dtype dtype, float* residual_table,
                           const int64_t* rows, int64_t U, int64_t D, int64_t R, int64_t k, int32_t block,
                           const gc_buf* out, void* hip_stream);

/* Aggregate of W workers' row-sparse buffers (as gc_compress_rows writes them: indices are table
 * positions row * D + column) over a given list of rows instead of the whole table: urows holds Ru
 * ascending unique row ids (DEVICE memory, int64) that contain every row any buffer touches, and
 * out (Ru * D fp32, fully overwritten) receives out[r * D + c] = sum over w, in worker order and in
 * fp32, of worker w's decoded value at table position urows[r] * D + c - what gc_decompress_sum
 * would leave in those rows of the dense table. staleness: W host entries or NULL (Eq. 12, as in
 * gc_decompress_sum_weighted). Ru * D < 2^32. A pair whose row is missing from urows is reported by
 * gc_sync_status() as GC_ERR_INVALID_ARG (the output is then unspecified). */
gc_status gc_decompress_sum_rows(gc_ctx* ctx, const gc_buf* bufs, int32_t W, const int64_t* urows, int64_t Ru,
                                 int64_t D, const int32_t* staleness, float* out, void* hip_stream);

/* Dense codes with error feedback: every entry is sent, so nothing is selected and there is no
 * index list. With GC_CODEC_SIGN1 this is the paper's 1-bit quantizer (Sec. III.B, Eq. 10: the signs
 * and one scale derived from the l1 norm) applied to the whole accumulated gradient, with the residual
 * of Eq. 11 feeding what the signs lose into the next step:
 *   acc = residual + grad;  per block of `block` consecutive ELEMENTS: scale and codes exactly as
 *   gc_compress computes them for a block of kept values;  residual = acc - decoded value.
 * The codes, scales and residual equal, bit for bit, those of gc_compress with k = n.
 * q: gc_num_code_bytes(n, block, codec) bytes; scales: gc_num_scales(n, block) fp32. block <= 8192
 * (GC_ERR_UNSUPPORTED beyond). Non-finite input is reported by gc_sync_status(). */
gc_status gc_compress_dense(gc_ctx* ctx, const void* grad, gc_dtype dtype, float* residual, int64_t n,
                            int32_t block, gc_codec codec, void* q, float* scales, void* hip_stream);

/* Aggregate of W workers' dense codes (Eq. 8 without the 1/P): out[i] = sum over w = 0..W-1, in that
 * order and in fp32, of worker w's decoded value at i; with `staleness` (W host entries in [0, 2^24],
 * or NULL) each term is first divided by 1 + staleness[w] (Eq. 12). q, scales: host arrays of W device
 * pointers, laid out as gc_compress_dense writes them. `out` (n fp32) is fully overwritten. */
gc_status gc_decompress_sum_dense(gc_ctx* ctx, const void* const* q, const float* const* scales, int32_t W,
                                  int32_t block, gc_codec codec, const int32_t* staleness, float* out,
                                  int64_t n, void* hip_stream);

/* The same aggregate applied at once (Eq. 9): theta[i] <- theta[i] - fl32(step * S[i]) for every i,
 * `step` standing for eta / P (0 <= step, finite). theta: n fp32, updated in place. */
gc_status gc_decompress_apply_dense(gc_ctx* ctx, const void* const* q, const float* const* scales, int32_t W,
                                    int32_t block, gc_codec codec, const int32_t* staleness, float* theta,
                                    float step, int64_t n, void* hip_stream);

/* Wait for `hip_stream` and return GC_ERR_NONFINITE if any compress call since
 * the last gc_sync_status() saw Inf/NaN among its kept entries (GC_ERR_INVALID_ARG if a
 * gc_compress_rows call saw a bad row id), else GC_OK. */
gc_status gc_sync_status(gc_ctx* ctx, void* hip_stream);

/* Counters of the most recent compress call; call after gc_sync_status(). */
gc_status gc_last_stats(gc_ctx* ctx, gc_stats* stats);

/* Per-kernel timing with HIP events recorded on the caller's stream around each
 * launch. gc_profile_enable(ctx, 1) starts a fresh recording of every kernel, 2 of the
 * streaming pass of gc_compress only (two event records per call), 0 stops; gc_profile_read
 * waits for the recorded events and returns, for kernel `id` in
 * [0, gc_profile_num_kernels()), the summed duration in milliseconds and the
 * number of launches since recording started. */
gc_status gc_profile_enable(gc_ctx* ctx, int32_t on);
int32_t gc_profile_num_kernels(void);
const char* gc_profile_kernel_name(int32_t id);
gc_status gc_profile_read(gc_ctx* ctx, int32_t id, double* total_ms, int64_t* launches);

/* Tuning knobs; the defaults are chosen for MI355X and results never depend on them.
 *   "main_lds_pad"  bytes of dynamic LDS requested by the streaming pass, used only to bound how
 *                   many of its workgroups share a compute unit (0..65536; default 16384).
 *   "dense_lds_pad" the same for the dense coder (0..65536, or -1: chosen by block size and code; default -1).
 *   "dense_wave_block"  dense coder: blocks of up to this many elements are held by one wavefront,
 *                   larger ones by a workgroup (0..2048; default 1024).
 *   "dec_large_tile"  the aggregate's output tile held in LDS by one wavefront: 16384 floats (1),
 *                   4096 floats (0), or chosen from the vector's length and filling (-1; default).
 *   "dec_fused"     the aggregate as one kernel that reads the workers' lists tile by tile (1), as two
 *                   kernels with a packed record stream in between (0), or chosen from the number of
 *                   workers and how the output tiles are filled (-1; default).
 *   "dec_fused_tile"  the one-kernel aggregate's launch shape: two workgroups per compute unit whose
 *                   wavefronts prepare a range of tiles together and then sum it (1: for crowded
 *                   tiles), one workgroup with two wavefronts that only prepare the next range (0: for
 *                   thinly filled tiles), or chosen from the filling and the number of workers (-1; default).
 *   "apply_dense_min"  fused apply: an output tile with at least this many pairs per 4096 floats is
 *                   read and rewritten whole instead of position by position (1..2^30; default 128).
 * Unknown names or out-of-range values return GC_ERR_INVALID_ARG. */
gc_status gc_set_option(gc_ctx* ctx, const char* name, int64_t value);

const char* gc_status_string(gc_status s);

#ifdef __cplusplus
}
#endif
#endif /* GRADCOMP_H */
