/*
 * kvprefetch -- paged-KV decode attention with asynchronous KV-block prefetch
 * for AMD MI355X (gfx950 / CDNA4).  C ABI.
 *
 * The operation is the attention decode step the paper accelerates (Section 3.1,
 * "Prefetch KV Blocks"): every new token's query attends over its sequence's
 * KV cache, which lives in fixed-size KV blocks located through a block table.
 * Algorithm 1 of the paper adds, before the compute on the current block, an
 * asynchronous fetch of the block the same wave will consume next; here that is
 * the `prefetch_distance` argument (0 = the baseline flow of Figure 2a, k >= 1 =
 * the fetch of the tile k iterations ahead is in flight while the current one
 * is computed, Figure 2b generalised).  Prefetching changes no result.
 *
 * All tensor arguments are DEVICE memory owned by the caller.  The library
 * enqueues kernels on `stream` and returns without synchronising; it allocates
 * nothing and keeps no pointer after return except the registered workspace.
 * State is kept per device (the device current at the call): workspace, the slices
 * of it that streams hold, the side stream of the layer stack.  The tuning and
 * comparison switches (kv_decode_set_waves_per_cu, _variant, _l2_touch, _xcd_skew)
 * and the two measurement aids (kv_profile_*, kv_decode_set_worker_trace) are
 * process-wide: they exist for benchmarks and tests, and a value set by one caller
 * is seen by every later call.
 *
 * Every entry point returns a kv_status; kv_last_error() gives the text of the
 * last failure on the calling thread.  No C++ exception crosses this boundary.
 */
#ifndef KVPREFETCH_H
#define KVPREFETCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KV_OK = 0,
    KV_ERR_INVALID = 1,     /* null pointer, rank / shape / stride / dtype mismatch, bad scalar */
    KV_ERR_UNSUPPORTED = 2, /* head_dim, block_size, dtype or group size the kernels do not cover */
    KV_ERR_HIP = 3,         /* a HIP runtime call failed; text from hipGetErrorString */
    KV_ERR_WORKSPACE = 4    /* split-KV workspace missing or too small */
} kv_status;

typedef enum { KV_F16 = 0, KV_BF16 = 1, KV_I32 = 2, KV_F32 = 3, KV_FP8_E4M3 = 4 /* OCP FP8 E4M3 codes, one byte */ } kv_dtype;

/* A device tensor: base pointer, element type, rank, extents and strides (in elements). */
typedef struct kv_tensor {
    void*   data;
    int32_t dtype; /* kv_dtype */
    int32_t ndim;
    int64_t shape[5];
    int64_t stride[5];
} kv_tensor;

/*
 * Paged decode attention (paper Section 3.1; Algorithm 1 for the prefetch order).
 *
 *   out[b,h,:] = sum_t softmax_t( scale * q[b,h,:] . K_b[t,:] ) * V_b[t,:],  t < context_lens[b]
 *   K_b[t,:]   = k_cache[ block_tables[b, t / block_size], h / (Hq/num_kv_heads), t % block_size, : ]
 *
 *   q            [B, Hq, d]                 f16 | bf16, last stride 1
 *   k_cache      [NBLK, Hkv, block_size, d] same dtype; the [block_size, d] tile of one
 *   v_cache      [NBLK, Hkv, block_size, d] (block, head) is dense (the paper's M_block, Eq. 1)
 *   block_tables [B, MB] int32, last stride 1.  Only entries [b, 0 .. ceil(n_b/block_size)-1]
 *                are read; ids are clamped to [0, NBLK) before use.
 *   context_lens [B] int32, dense.  n_b <= 0 gives a zero output row; n_b is clamped to
 *                MB * block_size.  Cache slots at t >= n_b are never used.
 *   out          [B, Hq, d] same dtype as q, last stride 1, rounded to nearest even.
 *   scale        multiplies the logits (1/sqrt(d) in the tests).
 *   prefetch_distance  0 .. KV_MAX_PREFETCH_DISTANCE, or KV_PREFETCH_AUTO.
 *   stream       hipStream_t, NULL = the default stream.
 *
 * Supported: d in {64, 128}, block_size in {16, 32}, Hq/Hkv in 1..16.  Every call needs the
 * registered workspace below.
 */
#define KV_MAX_PREFETCH_DISTANCE 4
/* prefetch_distance value that lets the library choose: the distance (and the occupancy that goes with it) measured
 * fastest on this chip for the cache type: 2 for 16-bit caches, 1 for kv_decode_attn_kv8. */
#define KV_PREFETCH_AUTO (-1)
int kv_decode_attn(const kv_tensor* q, const kv_tensor* k_cache, const kv_tensor* v_cache,
                   const kv_tensor* block_tables, const kv_tensor* context_lens, kv_tensor* out,
                   float scale, int num_kv_heads, int block_size, int prefetch_distance,
                   void* stream);

/*
 * Debugging aid, not for the hot path: the attention calls cannot report bad DATA (that would need
 * a synchronisation), they clamp instead.  This call waits for `stream`, copies block_tables and
 * context_lens to the host and checks what the kernels would otherwise clamp silently: every
 * context length in 0 .. MB * block_size, and every block id a sequence actually uses (entries
 * [b, 0 .. ceil(n_b / block_size) - 1]; the rest of a row may hold anything) in 0 .. num_blocks - 1.
 * KV_OK, or KV_ERR_INVALID with the first offending entry named in kv_last_error().  Allocates host
 * memory.
 */
int kv_validate_inputs(const kv_tensor* block_tables, const kv_tensor* context_lens, int num_blocks,
                       int block_size, void* stream);

/*
 * Measurement aid: the fetch stream of kv_decode_attn with the arithmetic left out.  Same
 * arguments and checks, same worker ranges, block-table lookups and asynchronous tile fetches at
 * the same prefetch_distance and occupancy; nothing is read back from LDS and nothing is written
 * (out is untouched, no merge kernel runs).  Its duration is what the memory system takes for
 * exactly this access pattern: the ceiling the attention kernel's roofline fraction is read
 * against.  Timed by kv_profile_enable like the main kernel.  16-bit caches only.
 */
int kv_decode_fetch_probe(const kv_tensor* q, const kv_tensor* k_cache, const kv_tensor* v_cache,
                          const kv_tensor* block_tables, const kv_tensor* context_lens, kv_tensor* out,
                          float scale, int num_kv_heads, int block_size, int prefetch_distance, void* stream);

/*
 * The same operation on an 8-bit KV cache (not in the paper: its Eq. 1 has the element size b as
 * a parameter, and halving b halves the bytes the kernel is bound by).  k_cache and v_cache hold
 * OCP FP8 E4M3 codes (dtype KV_FP8_E4M3, one byte per element, same [NBLK, Hkv, bs, d] layout
 * with the [bs, d] tile dense and outer strides multiples of 16); the values attended to are
 *     K = k_scale * e4m3(k_cache),   V = v_scale * e4m3(v_cache)      (one positive scale per tensor),
 * q and out stay f16 or bf16.  The kernel fetches the 8-bit tiles as they are, widens them to
 * q's type on the way to the matrix cores (exactly: both 16-bit types hold every E4M3 value) and
 * proceeds as kv_decode_attn; k_scale is folded into the softmax scale, v_scale into the normalisation.
 * Everything else (arguments, errors, workspace, prefetch_distance) as kv_decode_attn.
 */
int kv_decode_attn_kv8(const kv_tensor* q, const kv_tensor* k_cache, const kv_tensor* v_cache,
                       const kv_tensor* block_tables, const kv_tensor* context_lens, kv_tensor* out,
                       float scale, float k_scale, float v_scale, int num_kv_heads, int block_size,
                       int prefetch_distance, void* stream);

/*
 * Layer-stack harness: for l = 0 .. num_layers-1
 *     y      = x . weights[l]                 (bf16 in, fp32 accumulate, bf16 out -> gemm_out)
 *     q_l    = y[:, 0 : Hq*d] viewed [B, Hq, d]  (or q[l] when q != NULL: then y is unused by attention)
 *     outs[l] = kv_decode_attn(q_l, k_caches[l], v_caches[l], block_tables, context_lens, ...)
 * The GEMM is the compute window between two attention calls.  With
 * cross_layer_prefetch = 1 the leading KV tiles of layer l (the first tiles of every
 * worker's range) are touched on a side stream while GEMM_l, the kernel between
 * attention_{l-1} and attention_l, runs, so they sit in the memory-side cache when
 * attention_l starts; results do not depend on it.  The paper prefetches only inside
 * the attention kernel (next iteration, Section 3.1); the cross-layer form is this
 * repository's harness.  Every layer's arguments are checked before the first kernel is
 * enqueued: a call that returns an error has enqueued nothing.
 *
 *   x        [B, K] bf16, rows dense;  gemm_out [B, N] bf16, rows dense, N >= Hq*d when q == NULL
 *   weights[l] bf16, one of
 *            [K, N] row-major;
 *            [N/128, K, 128] tile-packed (column tile t holds W[:, 128t : 128t+128] as one contiguous run);
 *            [N/64, K/32, 4, 64, 8] in matrix-core operand order,
 *                Wp[t][ks][nb][l][j] = W[32 ks + 8 (l / 16) + j][64 t + 16 nb + l % 16],
 *            the form the kernel streams fastest (HBM straight into registers); it needs K of 1024, 2048,
 *            4096 or 8192 and a workspace of kv_layerstack_workspace_bytes()
 *   q, k_caches, v_caches, outs: arrays of num_layers tensor pointers (host arrays of
 *   host structs naming device memory).  Supported GEMM shapes: B <= 128, K % 128 == 0,
 *   N % 128 == 0.
 */
int kv_decode_layerstack(int num_layers, const kv_tensor* x, const kv_tensor* const* weights,
                         kv_tensor* gemm_out, const kv_tensor* const* q,
                         const kv_tensor* const* k_caches, const kv_tensor* const* v_caches,
                         const kv_tensor* block_tables, const kv_tensor* context_lens,
                         kv_tensor* const* outs, float scale, int num_kv_heads, int block_size,
                         int prefetch_distance, int cross_layer_prefetch, void* stream);

/*
 * Split-KV workspace (the block index range [s, e) that Algorithm 1 takes as input lets a
 * worker own part of a sequence; the pieces of a sequence that several workers share are
 * merged by a second kernel).  Bytes that are enough for any one call with these extents: a
 * fixed bound, 4096 bytes of words the dense layer of the layer stack uses, then two partial
 * pieces of min(Hq, 16) rows of (d + 4) floats for each of at most 4096 workers (69 MB at d 128,
 * Hq >= 16).  0 for unsupported extents.  What a call really takes is two pieces of Hq/Hkv rows
 * for each of its workers (compute units x waves per compute unit): 2 MB for 32 / 8 heads at
 * two waves on 256 compute units.
 * kv_layerstack_workspace_bytes: what kv_decode_layerstack needs when weights are in operand
 * order: the same plus two fp32 partial tiles of 128 x 128 per 128 columns of the dense layer
 * (its two halves of K meet there); gemm_n = columns of the dense layer.
 */
size_t kv_decode_workspace_bytes(int B, int Hq, int d, int max_context, int block_size);
size_t kv_layerstack_workspace_bytes(int num_q_heads, int head_dim, int gemm_n);

/*
 * Register caller-owned device scratch for later calls on the CURRENT device (any thread;
 * one registration per device).  NULL/0 unregisters.  While registered the memory belongs to the
 * library, which hands it out in slices: the first call on a stream takes a slice of the size it
 * needs from the unused end, later calls on that stream reuse it (or take a larger one), so
 * calls enqueued on different streams never share scratch and may overlap in time.  A call that
 * finds too little left returns KV_ERR_WORKSPACE and enqueues nothing; registering (the same or
 * another buffer) releases every slice, which is only safe once earlier calls have completed.
 * Calls on ONE stream share their slice, in stream order; a captured graph keeps the slice of
 * the stream it was captured on, so replays of it must not overlap each other or other work of
 * that stream.
 */
int kv_decode_set_workspace(void* dev_ptr, size_t bytes);

/*
 * kv_decode_attn for callers that cannot allocate and have no workspace to register: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * checks, kernels and results as kv_decode_attn; the split-KV scratch is a fixed array of
 * KV_NOALLOC_SCRATCH_BYTES inside the library's device image (every device the library runs on
 * holds it until the process ends) instead of the registered workspace.  The call allocates
 * nothing and frees nothing, on the host side of HIP or the device; the first call on a device
 * looks up the array's address there, later calls read it from a table.  A launch whose pieces
 * (workers x 2 x Hq/Hkv rows of (d + 4) floats) exceed the array returns KV_ERR_WORKSPACE with
 * the sizes in kv_last_error() and enqueues nothing: every automatic waves-per-compute-unit
 * choice on 256 compute units fits, 16 waves with 16 query heads per kv head does not.  Every
 * call on a device uses that device's one array, whatever the stream: calls that overlap in time
 * on one device race, calls in stream order do not.  Nothing in the array has to start at zero
 * (the merge kernel reads only the pieces the same call's main kernel wrote), so none of it is
 * cleared.
 */
#define KV_NOALLOC_SCRATCH_BYTES (32u << 20)
int kv_decode_attn_noalloc(const kv_tensor* q, const kv_tensor* k_cache, const kv_tensor* v_cache,
                           const kv_tensor* block_tables, const kv_tensor* context_lens, kv_tensor* out,
                           float scale, int num_kv_heads, int block_size, int prefetch_distance,
                           void* stream);

/*
 * Persistent waves (workers) per compute unit, 1 .. 16; 0 restores the automatic choice, which
 * aims at 32-48 KB of KV in flight per compute unit: 6 waves at prefetch distance 0 or 1 and 2
 * waves at distance 2 or more for head_dim 128, 8 and 4 waves for head_dim 64.
 * Each worker holds (prefetch_distance + 1) stages of LDS (a tile pair of 8 KB and the query image of
 * a unit, 4 KB, at head_dim 128; 4 KB + 2 KB at 64), so the number in effect is capped by the 160 KB
 * of a compute unit (Eq. 2 re-derived for LDS as the prefetch target: bytes in flight per CU = tile
 * pair x prefetch_distance x waves);
 * kv_decode_get_waves_per_cu returns the number a call with that distance and head_dim would use
 * (for the kernel variant in effect, see kv_decode_set_variant).
 */
int kv_decode_set_waves_per_cu(int waves);
int kv_decode_get_waves_per_cu(int prefetch_distance, int head_dim);
/* The same for a given number of query heads per kv head (1 .. 16), on which the LDS of a worker of the
 * two-phase variant depends (kv_decode_get_waves_per_cu assumes 16 there); 0 for invalid arguments. */
int kv_decode_get_waves_per_cu_for(int prefetch_distance, int head_dim, int q_heads_per_kv_head);
/* The same for kv_decode_attn_kv8 (stages of the same bytes, holding 32 tokens; twice the arithmetic
 * per byte, so more waves: at head_dim 128 6 waves at distance 0 and 3 with a look-ahead, at head_dim 64
 * 8 waves, fewer where the LDS caps them, and above four an even number). */
int kv_decode_get_waves_per_cu_kv8(int prefetch_distance, int head_dim);

/*
 * Kernel form of kv_decode_attn (and of the layer stack's attention) on 16-bit caches.
 * KV_VARIANT_ONE_PASS (default): online softmax, the K and the V tile of 16 tokens fetched and
 * consumed together.  KV_VARIANT_TWO_PHASE: the form of the kernel the paper patches (its Sections
 * 3.1 and 3.2): per chunk of up to 512 tokens first all logits (next K tile prefetched during the
 * current one's product), kept in LDS, then the weights applied to the V tiles (next V tile
 * prefetched likewise); prefetch_distance d keeps 2 d single tiles in flight, the bytes of the
 * one-pass form.  Same work mapping, workspace and results up to rounding; each worker holds
 * (2 d + 1) tiles plus 32 KB of logits in LDS, which caps the waves per compute unit.
 * kv_decode_attn_kv8 ignores the setting.
 */
enum { KV_VARIANT_ONE_PASS = 0, KV_VARIANT_TWO_PHASE = 1 };
int kv_decode_set_variant(int variant);

/*
 * Comparison mode: the paper's own mechanism, prefetch into L2 (its Section 3.2), in place of the
 * LDS ring.  With tiles > 0, calls of kv_decode_attn (and the layer stack) with prefetch_distance 0
 * launch every worker with a second wave that walks the same range and touches the K and V tiles
 * ahead of it into L2 (one dword per 128-byte line), in groups of `tiles` tiles and at most two
 * groups ahead of the worker; the worker itself fetches, waits and computes as at distance 0 and
 * finds its lines in L2.  Results are those of distance 0.  0 (the default) switches it off;
 * 0 .. 8.  Calls with another prefetch_distance, the two-phase variant and kv_decode_attn_kv8
 * ignore it.
 */
int kv_decode_set_l2_touch(int tiles);

/*
 * Comparison mode for the cache-policy study (the paper's remark on the eviction priority of prefetched
 * data, Section 3.3): KV_FETCH_NON_TEMPORAL (default) marks every KV fetch, and every weight load of the
 * layer stack's dense layer in operand order, non-temporal: the data is used once and should not displace
 * anything in L2 or the memory-side cache.  KV_FETCH_PLAIN drops the hint, as the "before" of that
 * comparison; it is built for the benchmark shapes only (kv_decode_attn on bf16, head_dim 128,
 * prefetch_distance 0 or 2, one-pass variant; dense layer with K = 4096), other calls return
 * KV_ERR_UNSUPPORTED while it is set.  Results do not depend on it.
 */
enum { KV_FETCH_NON_TEMPORAL = 0, KV_FETCH_PLAIN = 1 };
int kv_decode_set_fetch_policy(int policy);

/*
 * Skew of the workers' shares of the tile space between the even and the odd XCD of every XCD
 * pair, in 1/1024: worker w gets 1024 + skew parts when w is even and 1024 - skew when it is odd
 * (workgroups go to the XCDs round-robin; under load the odd XCD of a pair delivers about 3 % less
 * bandwidth).  0 gives equal shares; 0 .. 256; default 10.  Results depend on it only through
 * where units are cut (rounding of the merge), like on the worker count.
 */
int kv_decode_set_xcd_skew(int per_1024);

/*
 * Timing of the main attention kernel with HIP events on the call's own stream (the paper
 * reports the attention kernel's duration, Table 2).  kv_profile_enable(n, every) creates
 * events for n samples (host-side allocation, not on the timed path; n = 0 frees them); while
 * enabled, every `every`-th kv_decode_attn call records one event before and one after its
 * main kernel (an event pair costs a few microseconds of stream time, hence the sampling).
 * kv_profile_read waits for the recorded calls, returns the summed kernel durations in
 * milliseconds and the number of calls, and rearms the same events; kv_profile_read_each does
 * the same and returns every sample's duration (main_ms holds `capacity` floats; more samples
 * than that is an error and nothing is consumed), for medians.  Calls from several threads
 * share one slot counter under a mutex.
 */
int kv_profile_enable(int max_calls, int every);
int kv_profile_read(double* main_ms_sum, int* calls);
int kv_profile_read_each(float* main_ms, int capacity, int* calls);

/*
 * Per-worker timeline of the main attention kernel (where inside a launch the time goes: the
 * paper's Table 1 asks that of its baseline kernel with a profiler; this is the kernel's own
 * account).  While device memory is registered here, every persistent worker w of a launch with
 * at most bytes / 32 workers writes four 64-bit words at dev_ptr + 32 w: the constant 100 MHz
 * clock at entry, after it has located its range, at exit, and a word whose low 32 bits are the
 * number of tiles it processed, whose bits 32..35 are the XCD (XCC_ID) it ran on and whose bits
 * 40..55 are the time from "range located" until its first tile pair had landed, in clock ticks of
 * 10 ns (saturating; kv_decode_attn's one-pass kernel only, zero elsewhere): the latency the
 * cross-layer touch of the layer stack is meant to shorten.
 * NULL/0 unregisters.  The caller owns the memory and reads it after synchronising;
 * launches with more workers than fit leave it untouched.  Costs two clock reads per worker.
 */
int kv_decode_set_worker_trace(void* dev_ptr, size_t bytes);

/* Text of the last error on this thread; never NULL. */
const char* kv_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int kv_version(void);

/* Eq. 1 of the paper: bytes of one K (or V) block of one head. */
size_t kv_block_bytes(int elem_bytes, int head_dim, int block_size);

/* Eq. 2 of the paper: bytes of the blocks one loop iteration of the whole grid touches;
 * units_per_wg is the number of waves of a workgroup (N_thread / 32 in the paper). */
size_t kv_iter_working_set_bytes(size_t block_bytes, int units_per_wg, int H, int B);

/*
 * The attention kernels' partition of the flat tile space (all tiles of all (sequence, kv head)
 * units in order; Algorithm 1's block range [s, e) of a warp becomes one contiguous range per
 * persistent wave), computed on the host by the code the kernels run.  `tiles` >= 1 tiles are cut
 * among min(workers, tiles) workers; xcd_skew as in kv_decode_set_xcd_skew.
 * kv_worker_range: first tile and end (one past the last) of worker's range; status.
 * kv_worker_of_tile: the worker whose range holds `tile`, or -1 for invalid arguments.
 */
int kv_worker_range(int64_t tiles, int workers, int xcd_skew, int worker, int64_t* first, int64_t* end);
int kv_worker_of_tile(int64_t tiles, int workers, int xcd_skew, int64_t tile);

#ifdef __cplusplus
}
#endif
#endif /* KVPREFETCH_H */
