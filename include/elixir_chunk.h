/*
 * elixir_chunk.h -- C ABI of libelixir_chunk.so
 *
 * The chunked mixed-precision AdamW step of Elixir (arXiv 2212.05339) on one
 * AMD MI355X (gfx950).  Parameters are flattened into fixed-length 1-D chunks
 * (paper Sec. 3 "Chunk"); each low-precision parameter chunk is paired with an
 * optimizer chunk holding the fp32 master weight and the two Adam moments on
 * the same device (paper Sec. 4.1); one optimizer update consumes a gradient
 * chunk and its optimizer chunk and leaves the low-precision parameters for
 * the next forward pass (paper Sec. 2 "Mixed Precision Training").  Chunks the
 * plan keeps in host memory are moved to the GPU and back on side streams so
 * that transfers overlap with work on resident chunks (paper Sec. 4.3).
 *
 * General rules
 *   - Every function returns an int status: ELIXIR_OK (0) or a negative code;
 *     elixir_last_error() gives a per-thread message for the last failure.
 *     Nothing throws across this boundary.
 *   - "d_" / device pointers must be accessible from the GPU that owns the
 *     stream; "h_" / host pointers are ordinary or pinned host memory as stated.
 *   - Lengths and offsets are counted in ELEMENTS (int64_t) unless named *_bytes.
 *   - bf16 values are passed as their 16-bit patterns (uint16_t).
 *   - Every GPU operation is enqueued on the caller's stream and returns
 *     without waiting for it; no entry point synchronises the device except
 *     elixir_ctx_destroy (elixir_stream_synchronize waits for the stream it is given; elixir_offload_copy_streams,
 *     a set-up call, waits for the probes it issues).  elixir_stream_t is a hipStream_t (NULL = the
 *     default stream).  The caller's current device must be the one that owns
 *     the stream and buffers.
 *   - The caller owns every buffer it passes in.  The library owns only what
 *     elixir_ctx_create and elixir_host_alloc allocate.  No other entry point
 *     allocates device or pinned memory that outlives the call.
 *   - Pointers must be naturally aligned for their element type.  Whole
 *     chunks from any allocator are aligned far beyond what the vector kernels
 *     need (8 bytes for the AdamW state, 16 for reduce and pack); slices at
 *     other alignments take a one-element-per-thread kernel with identical
 *     results.
 */
#ifndef ELIXIR_CHUNK_H
#define ELIXIR_CHUNK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ELIXIR_OK        0
#define ELIXIR_EINVAL   (-1) /* NULL where a pointer is required, negative length, bad enum, overlapping slices ... */
#define ELIXIR_EALIGN   (-2) /* pointer not naturally aligned for its element type */
#define ELIXIR_ENOSLOT  (-3) /* every staging slot is held by a chunk that has not been evicted yet */
#define ELIXIR_EHIP     (-4) /* a HIP runtime call failed; the message names it */
#define ELIXIR_ESTATE   (-5) /* call out of order (slot not prefetched, slots not registered ...) */
#define ELIXIR_ECAP     (-6) /* more chunks / elements than the context or an output array was sized for */

typedef void* elixir_stream_t;          /* a hipStream_t */
typedef struct elixir_ctx elixir_ctx;   /* opaque */

/* Hyper-parameters of one AdamW step.  step is 1-based (the first update has step = 1). */
typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    int64_t step;
} elixir_adam_hparams;

/* Chunk grouping policies for elixir_layout_plan. */
enum {
    ELIXIR_LAYOUT_NEXT_FIT = 0,  /* the paper's grouping (App. A.2): one current chunk */
    ELIXIR_LAYOUT_FIRST_FIT = 1, /* earliest chunk with room */
    ELIXIR_LAYOUT_DENSE = 2      /* parameters may straddle chunk boundaries */
};

/* Low-precision formats of gradients and parameter copies (16-bit patterns either way). */
enum {
    ELIXIR_LOWP_BF16 = 0, /* what the benchmark configurations use */
    ELIXIR_LOWP_FP16 = 1  /* IEEE binary16, the paper's format (Sec. 2 "Mixed Precision Training") */
};

/* Per-thread message describing the last non-OK status returned on this thread ("" if none). */
const char* elixir_last_error(void);

/*
 * Context: device workspace for the norm reduction (one double per reduction
 * block) and the bookkeeping of the offload pipeline.  max_chunk_elems and
 * max_chunks bound what elixir_chunk_grad_norm accepts.  The context is bound
 * to HIP device `device`.  Not thread-safe: use one context per host thread.
 * elixir_ctx_destroy waits for the device, frees the workspace and events
 * (not the caller's slots or host blocks).
 */
int elixir_ctx_create(elixir_ctx** out, int device, int64_t max_chunk_elems, int max_chunks);
int elixir_ctx_destroy(elixir_ctx* ctx);

/*
 * Chunk layout (host only, integers).  Paper App. A.2: walk the parameters in
 * their order of use, keep one current chunk, append a parameter if it fits,
 * otherwise close the chunk and open a new one (NEXT_FIT).  A parameter longer
 * than chunk_elems starts at offset 0 of a fresh chunk and runs through
 * ceil(numel/chunk_elems) consecutive chunks; the rest of its last chunk stays
 * open.  FIRST_FIT searches every chunk, oldest first; DENSE keeps one running
 * position so that only the last chunk is padded.  Every start is rounded up to
 * a multiple of align_elems (>= 1, must divide chunk_elems).
 *   in : numel[T] (>= 0), chunk_elems (> 0), policy, align_elems
 *   out: chunk_id[T], offset[T]  -- parameter i occupies the linear element
 *        range [chunk_id[i]*chunk_elems + offset[i], +numel[i]);
 *        *n_chunks; valid_len[0..*n_chunks) = elements in use per chunk
 *        (valid_len may be NULL; otherwise valid_cap is its capacity and
 *        ELIXIR_ECAP is returned, with *n_chunks set, if it is too small).
 */
int elixir_layout_plan(const int64_t* numel, int T, int64_t chunk_elems, int policy, int64_t align_elems,
                       int64_t* chunk_id, int64_t* offset, int64_t* n_chunks, int64_t* valid_len,
                       int64_t valid_cap);

/*
 * Pack / unpack (paper Fig. 3, left panel: every parameter's data sits in a
 * slice of its parameter chunk).  Bit copies, elem_size 2 or 4 bytes.
 *   pack  : d_chunk[offset[i] + k] = tensors[i][k] for k < numel[i]; every
 *           element of the chunk not covered by a slice is set to zero bits.
 *   unpack: tensors[i][k] = d_chunk[offset[i] + k].
 * tensors is a HOST array of T device pointers; numel/offset are host arrays.
 * Slices must lie inside [0, chunk_elems) and must not overlap (ELIXIR_EINVAL).
 * A parameter that spans several chunks is passed piecewise by the caller.
 */
int elixir_chunk_pack(void* d_chunk, int64_t chunk_elems, int elem_size, const void* const* tensors,
                      const int64_t* numel, const int64_t* offset, int T, elixir_stream_t stream);
int elixir_chunk_unpack(const void* d_chunk, int64_t chunk_elems, int elem_size, void* const* tensors,
                        const int64_t* numel, const int64_t* offset, int T, elixir_stream_t stream);

/*
 * The same for a whole parameter set in one call (a handful of launches instead of one per chunk: slices whose two
 * addresses are 16-byte aligned travel as the rows of a 2-D grid, up to 336 per launch), taking the layout plan as
 * elixir_layout_plan returns it: tensor i occupies the linear element range
 * [chunk_id[i] * chunk_elems + offset[i], + numel[i]) of the chunk sequence d_chunks[0], d_chunks[1], ... (a HOST array
 * of n_chunks device pointers), so a tensor that is longer than the rest of its chunk continues at the start of the
 * next one and need not be passed piecewise.  pack zero-fills every element of every chunk that no tensor covers.
 * Same bits as the per-chunk calls.  Tensors must not overlap and must lie inside the n_chunks chunks (ELIXIR_EINVAL).
 */
int elixir_chunks_pack(void* const* d_chunks, int n_chunks, int64_t chunk_elems, int elem_size, const void* const* tensors,
                       const int64_t* numel, const int64_t* chunk_id, const int64_t* offset, int T, elixir_stream_t stream);
int elixir_chunks_unpack(const void* const* d_chunks, int n_chunks, int64_t chunk_elems, int elem_size, void* const* tensors,
                         const int64_t* numel, const int64_t* chunk_id, const int64_t* offset, int T, elixir_stream_t stream);

/*
 * Gradient reduction into the fp32 gradient chunk.  In the paper gradients are
 * reduced across ranks and the reduced chunk feeds the optimizer update (Sec. 2
 * "ZeRO", Fig. 3 right); with one GPU the reduction that remains is the sum
 * over micro-batches:
 *   d_grad_chunk[offset+k] = fl32( (accumulate ? d_grad_chunk[offset+k] : 0) + fl32(scale * bf16->fp32(d_grad_bf16[k])) )
 * for k < n, with separately rounded multiply and add (no fused multiply-add).
 * The caller guarantees offset + n does not exceed the chunk.
 */
int elixir_grad_reduce_into_chunk(float* d_grad_chunk, int64_t offset, const uint16_t* d_grad_bf16, int64_t n,
                                  float scale, int accumulate, elixir_stream_t stream);

/*
 * Global gradient L2 norm over the valid part of n_chunks fp32 gradient chunks
 * and the clipping coefficient derived from it (not in the paper; the usual
 * definition):  norm = sqrt(sum g^2),  coef = max_norm > 0 ? min(1, max_norm/(norm + 1e-6)) : 1.
 * The sum is taken in double precision over a fixed reduction tree, so the
 * result is bitwise reproducible from run to run.  grad_chunks and valid_len
 * are HOST arrays (device pointers / lengths).  *d_norm_out and
 * *d_clip_coef_out (either may be NULL) are DEVICE floats written on `stream`;
 * pass d_clip_coef_out as d_grad_scale to elixir_chunk_adam_step to clip
 * without a host round trip.  Uses the context's workspace: calls on one
 * context must be stream-ordered with each other.
 */
int elixir_chunk_grad_norm(elixir_ctx* ctx, const float* const* grad_chunks, const int64_t* valid_len,
                           int n_chunks, float max_norm, float* d_norm_out, float* d_clip_coef_out,
                           elixir_stream_t stream);

/*
 * elixir_chunk_grad_norm for callers that cannot allocate or hold a context: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments without the context, same kernels, bit-identical
 * results.  The partial sums go to a static array inside the library's device code (4 MiB on every GPU the library
 * runs on, held until the process ends) instead of a context's workspace; the call allocates and frees nothing, on
 * the device or the host.  Limits: n_chunks <= 512 (ELIXIR_ECAP beyond; chunk lengths are not limited), HIP devices
 * 0..63.  The array's device address is looked up once per device: by elixir_ctx_create for its device, else by the
 * first call on that device (make that first call outside a graph capture).  All calls on one GPU share the one
 * array: calls that overlap in time on the same GPU (different streams, different threads) race and give wrong
 * norms; order them on one stream or with events.  Nothing has to be cleared between calls: every slot that is read
 * is written first by the same call.
 */
int elixir_chunk_grad_norm_noalloc(const float* const* grad_chunks, const int64_t* valid_len, int n_chunks,
                                   float max_norm, float* d_norm_out, float* d_clip_coef_out, elixir_stream_t stream);

/*
 * The same norm taken directly over 16-bit gradient chunks.  The paper's gradient chunk IS a low-precision chunk (the
 * gradients take the place of the parameters in it, Sec. 4.1); with a single micro-batch nothing has to be summed in
 * fp32 first, and norm + update then move 2 + 28 bytes per element instead of 6 (widening pass) + 30.  Every element
 * is widened exactly and squared and summed in double over the same fixed tree:
 *   norm = |scale| * sqrt(sum g^2),   coef = max_norm > 0 ? min(1, max_norm/(norm + 1e-6)) : 1,
 *   *d_norm_out = norm,   *d_grad_scale_out = scale * coef
 * scale is the factor the stored gradients still have to be multiplied by (1/micro-batches, 1/ranks; 1 if none), so
 * *d_grad_scale_out is what the AdamW entry points take as d_grad_scale.  With fp16 gradients under loss scaling pass
 * scale = 1 and hand *d_norm_out to elixir_loss_scale_update (an Inf/NaN gradient gives a non-finite norm).
 * grad_chunks_lowp and valid_len are HOST arrays; chunk pointers need 2-byte alignment only.  Same workspace rule as
 * elixir_chunk_grad_norm.
 */
int elixir_chunk_grad_norm_lp(elixir_ctx* ctx, const uint16_t* const* grad_chunks_lowp, int lowp_format,
                              const int64_t* valid_len, int n_chunks, float scale, float max_norm, float* d_norm_out,
                              float* d_grad_scale_out, elixir_stream_t stream);

/*
 * The last pass of the reduction and the norm in one sweep.  elixir_grad_reduce_chunk_sumsq does what
 * elixir_grad_reduce_into_chunk_lp does for a WHOLE chunk (offset 0, chunk_elems elements, 16-byte aligned chunk,
 * 8-byte aligned gradients) and, from the values it is writing, leaves the chunk's sum of squares over its first
 * valid_len elements in the context's slots for chunk number chunk_index (< max_chunks).  After every chunk of the
 * step has gone through it (typically with the last micro-batch), elixir_chunk_grad_norm_finish(n_chunks) turns the
 * slots of chunks 0 .. n_chunks-1 into the norm and the clip coefficient exactly as elixir_chunk_grad_norm does --
 * without reading the gradients again (4 bytes per element saved).  Deterministic like the unfused path (its
 * summation tree differs, so the two norms may differ in the last bit).  The calls of one step share the context's
 * workspace and must use ONE stream: a reduction or the finish call that arrives on another stream than the
 * reductions since the last finish returns ELIXIR_ESTATE (use one context per stream).  Between steps, and for
 * elixir_chunk_grad_norm / _lp, ordering calls on different streams is the caller's business.
 */
int elixir_grad_reduce_chunk_sumsq(elixir_ctx* ctx, int chunk_index, float* d_grad_chunk, const uint16_t* d_grad_lowp,
                                   int lowp_format, int64_t chunk_elems, int64_t valid_len, float scale, int accumulate,
                                   elixir_stream_t stream);
int elixir_chunk_grad_norm_finish(elixir_ctx* ctx, int n_chunks, float max_norm, float* d_norm_out,
                                  float* d_clip_coef_out, elixir_stream_t stream);

/*
 * Fused AdamW over one chunk pair (paper Sec. 4.1: one optimizer update per
 * gradient chunk + optimizer chunk; Sec. 2: fp32 master rounded to the
 * low-precision parameters).  Adam (Kingma & Ba, Alg. 1) with decoupled weight
 * decay (Loshchilov & Hutter, Alg. 2), eps added after the bias correction of
 * sqrt(v).  For k < n, with s = d_grad_scale ? *d_grad_scale : 1 and t = hp->step:
 *   g = s * grad[k]
 *   p = master[k] * (1 - lr*wd)
 *   m = beta1*m[k] + (1-beta1)*g          v = beta2*v[k] + (1-beta2)*g*g
 *   p = p - lr * (m / (1-beta1^t)) / ( sqrt(v / (1-beta2^t)) + eps )
 *   master[k] = p;  exp_avg[k] = m;  exp_avg_sq[k] = v;  param_bf16[k] = round-to-nearest-even bf16(p)
 * Exactly one of d_grad_fp32 / d_grad_bf16 is non-NULL.  d_param_bf16 may be
 * NULL (no low-precision copy).  d_grad_scale is a DEVICE float or NULL.
 * d_param_bf16 may be EQUAL to d_grad_bf16: in the paper the gradient of a
 * parameter takes the place of the parameter in its low-precision chunk during
 * the backward pass (Sec. 4.1), so the update reads the gradients from the
 * parameter chunk and writes the new parameters over them (same speed, 2 bytes
 * per parameter saved).  This holds for every AdamW entry point of this header,
 * device and host; any other overlap between the arrays of a call is an error
 * of the caller and is not detected.
 * Arithmetic is fp32; algorithmic traffic is 28 bytes per element with bf16
 * gradients (2 + 12 read, 12 + 2 written), 30 with fp32 gradients.
 */
int elixir_chunk_adam_step(float* d_master, float* d_exp_avg, float* d_exp_avg_sq, const float* d_grad_fp32,
                           const uint16_t* d_grad_bf16, uint16_t* d_param_bf16, int64_t n,
                           const elixir_adam_hparams* hp, const float* d_grad_scale, elixir_stream_t stream);

/*
 * The same update for n_chunks chunk pairs in as few launches as possible (one
 * per 64 chunks): chunks much shorter than ~16Mi elements are launch-bound when
 * updated one call at a time.  All tables are HOST arrays of n_chunks entries;
 * the step constants and d_grad_scale are shared.  Exactly one of the two
 * gradient tables is non-NULL; d_param_bf16 may be NULL (no low-precision
 * copies).  Results are bit-identical to n_chunks calls of
 * elixir_chunk_adam_step.  Chunks must not overlap.
 */
int elixir_chunk_adam_step_multi(int n_chunks, float* const* d_master, float* const* d_exp_avg,
                                 float* const* d_exp_avg_sq, const float* const* d_grad_fp32,
                                 const uint16_t* const* d_grad_bf16, uint16_t* const* d_param_bf16, const int64_t* n,
                                 const elixir_adam_hparams* hp, const float* d_grad_scale, elixir_stream_t stream);

/*
 * Tiled optimizer chunk.  The paper's optimizer chunk holds the fp32 master weights and the Adam moments of one
 * chunk (Sec. 4.1) without saying how they are laid out.  Three separate arrays (the entry points above) make the
 * update read and write three streams far apart; interleaving them in tiles of ELIXIR_STATE_TILE elements,
 *   d_state = [ master tile | exp_avg tile | exp_avg_sq tile ] [ master tile | ... ] ...,
 * element e of the chunk at d_state[3*T*(e/T) + k*T + e%T] for k = 0, 1, 2 (T = ELIXIR_STATE_TILE), measured 2.5-3%
 * faster on MI355X.  A tiled chunk of n elements occupies elixir_state_tiled_len(n) = 3*T*ceil(n/T) floats; it is one
 * buffer, so a host-resident copy of it moves through the offload pipeline as any other block.
 *   elixir_state_tile / elixir_state_untile : flat arrays -> tiled buffer (positions past n in the last tile are
 *       zeroed) and back; bit copies, for set-up and checkpoints.
 *   elixir_chunk_adam_step_tiled_lp : elixir_chunk_adam_step_lp on a tiled chunk; bit-identical results.  d_state
 *       must be 8-byte aligned.
 *   elixir_chunk_adam_step_tiled_multi_lp : elixir_chunk_adam_step_multi_lp on tiled chunks (d_state is a HOST
 *       array of n_chunks tiled buffers).
 */
#define ELIXIR_STATE_TILE 4096
int64_t elixir_state_tiled_len(int64_t n);
int elixir_state_tile(float* d_state, const float* d_master, const float* d_exp_avg, const float* d_exp_avg_sq, int64_t n,
                      elixir_stream_t stream);
int elixir_state_untile(const float* d_state, float* d_master, float* d_exp_avg, float* d_exp_avg_sq, int64_t n,
                        elixir_stream_t stream);
int elixir_chunk_adam_step_tiled_lp(float* d_state, const float* d_grad_fp32, const uint16_t* d_grad_lowp,
                                    uint16_t* d_param_lowp, int lowp_format, int64_t n, const elixir_adam_hparams* hp,
                                    const float* d_grad_scale, const int32_t* d_skip, elixir_stream_t stream);

int elixir_chunk_adam_step_tiled_multi_lp(int n_chunks, float* const* d_state, const float* const* d_grad_fp32,
                                          const uint16_t* const* d_grad_lowp, uint16_t* const* d_param_lowp, int lowp_format,
                                          const int64_t* n, const elixir_adam_hparams* hp, const float* d_grad_scale,
                                          const int32_t* d_skip, elixir_stream_t stream);

/*
 * The step constants in device memory, so that one captured HIP graph replays step after step.  The entry points above
 * take the step number in `hp` and turn it into kernel arguments (lr/(1-beta1^t), 1/sqrt(1-beta2^t)): a graph captured
 * from them repeats that one step number.  Here the hyper-parameters, the number of steps done and the constants of the
 * current step live in a 64-byte DEVICE struct:
 *   elixir_adam_step_state_init    : one-thread kernel; copies hp and sets steps done = hp->step - 1.
 *   elixir_adam_step_state_advance : one-thread kernel; unless *d_skip (DEVICE flag, may be NULL) is non-zero, counts
 *       one step on and derives that step's constants in double precision, rounded once to fp32, as the host does
 *       for the other entry points.  Call it once per step, before the step's updates, on the same stream.
 *   elixir_chunk_adam_step_tiled_dev / _tiled_multi_dev : elixir_chunk_adam_step_tiled_lp / _tiled_multi_lp with the
 *       constants read from *d_step_state.  Results are those of the hp entry points for the same step number
 *       (bit-identical whenever the device's and the host's pow agree to the last bit of the rounded constants).
 * A graph that holds advance + the step's updates replays as steps t, t+1, t+2, ...; the host can read the struct
 * back to see the step count.  The struct must be 8-byte aligned.
 */
typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    int32_t reserved;
    int64_t step;     /* steps done so far */
    float consts[8];  /* constants of the current step, private to the library */
} elixir_adam_step_state;
int elixir_adam_step_state_init(elixir_adam_step_state* d_step_state, const elixir_adam_hparams* hp, elixir_stream_t stream);
int elixir_adam_step_state_advance(elixir_adam_step_state* d_step_state, const int32_t* d_skip, elixir_stream_t stream);
int elixir_chunk_adam_step_tiled_dev(float* d_state, const float* d_grad_fp32, const uint16_t* d_grad_lowp,
                                     uint16_t* d_param_lowp, int lowp_format, int64_t n,
                                     const elixir_adam_step_state* d_step_state, const float* d_grad_scale,
                                     const int32_t* d_skip, elixir_stream_t stream);
int elixir_chunk_adam_step_tiled_multi_dev(int n_chunks, float* const* d_state, const float* const* d_grad_fp32,
                                           const uint16_t* const* d_grad_lowp, uint16_t* const* d_param_lowp, int lowp_format,
                                           const int64_t* n, const elixir_adam_step_state* d_step_state,
                                           const float* d_grad_scale, const int32_t* d_skip, elixir_stream_t stream);

/*
 * Placement of the long-lived chunk buffers.  The paper allocates what lives as long as the run (optimizer states,
 * rCache blocks) once, before training (Sec. 3 "Pre-runtime Profiler", finding 2).  On MI355X where those buffers lie
 * relative to each other is worth 2-7% of the update's bandwidth: arrays that one kernel reads together (a chunk's
 * optimizer chunk, its gradient arrays, its fp32 gradient chunk) want to sit side by side in one allocation, arrays
 * that are only written (the low-precision parameter copies) somewhere else, and no two arrays a multiple of a few MiB
 * apart.  Host only, integers; allocates nothing.
 *   arrays[a] : one kind of per-chunk array: its size in bytes, how many of them a chunk has (e.g. several gradient
 *       sets), and its region (ELIXIR_ARENA_NEAR: laid out chunk after chunk, array after array, in region 0;
 *       ELIXIR_ARENA_FAR: the same in region 1).
 *   offset_out[c * K + k] : byte offset, from the start of its region, of the k-th array of chunk c, where k counts
 *       the arrays of a chunk in the order given (array 0's `count` instances, then array 1's, ...; K = sum of the
 *       counts).  Every offset is a multiple of 8192 and every array is followed by ELIXIR_ARENA_GAP_BYTES.
 *       offset_cap is the capacity of offset_out in entries (ELIXIR_ECAP if it is too small; region_bytes_out is set).
 *   region_bytes_out[2] : bytes the caller has to allocate for region 0 and region 1 -- two allocations, made as far
 *       apart in the address space as the caller can arrange (e.g. region 1 first, before other large allocations).
 */
#define ELIXIR_ARENA_GAP_BYTES ((4 << 20) + 8192)
enum { ELIXIR_ARENA_NEAR = 0, ELIXIR_ARENA_FAR = 1 };
typedef struct {
    int64_t bytes;
    int32_t count;
    int32_t region;
} elixir_arena_array;
int elixir_arena_plan(int n_chunks, const elixir_arena_array* arrays, int n_arrays, int64_t* offset_out,
                      int64_t offset_cap, int64_t* region_bytes_out);

/*
 * Offload pipeline for chunks whose optimizer chunk lives in host memory (the
 * paper keeps a searched number of chunks in CPU memory, Sec. 3 "Search
 * Engine", and overlaps chunk movement with computation by running it on
 * separate streams, Sec. 4.3).  Here the fp32 state of such a chunk is copied
 * into a device staging slot, updated by elixir_chunk_adam_step, and copied
 * back.
 *
 *   elixir_host_alloc / elixir_host_free : page-locked host memory.
 *   elixir_offload_register_slots : d_slots is a HOST array of n_slots device
 *       buffers of slot_bytes each, owned by the caller; replaces any earlier
 *       registration (ELIXIR_ESTATE while a slot is held).
 *   elixir_chunk_prefetch : picks a slot that is not held, makes h2d_stream
 *       wait until that slot's previous eviction has finished (and any eviction
 *       still on its way into h_block from another slot), enqueues the
 *       host-to-device copy of `bytes` (<= slot_bytes) from h_block and marks
 *       the slot held.  *slot_out receives the slot index.  ELIXIR_ENOSLOT if
 *       all slots are held.
 *   elixir_chunk_wait_ready : makes compute_stream wait for the slot's copy.
 *   elixir_chunk_evict : makes d2h_stream wait for the work enqueued so far on
 *       compute_stream, enqueues the device-to-host copy of `bytes` into
 *       h_block (h_block NULL: no copy, the slot is only released), and marks
 *       the slot free for the next prefetch.
 *   elixir_offload_copy_streams : set-up call; hands out the two copy streams of the pipeline.  They belong to the
 *       library, one pair per GPU, created by the first call and kept until the process ends (later calls verify the
 *       pair against their compute_stream and return it again); ctx only names the GPU.  The HIP runtime feeds all
 *       streams of a process through a few hardware queues (4 by default), and two streams that share one hold each
 *       other back whenever one of them waits: uploads and downloads then take turns (measured: 28 GB/s each way
 *       instead of 46-48), or kernels wait for block copies.  Which streams share a queue depends on how many streams
 *       the process has created, so the call measures it: it creates streams until two of them are seen to run beside
 *       compute_stream and beside each other (a marker on one stream must complete while a 64 MiB copy is still
 *       pending on the other), keeps those and destroys the rest; ELIXIR_ESTATE if there are no two among 12
 *       candidates.  Separate queues are necessary for uploads and downloads to overlap, not sufficient: after device
 *       memory has been freed (by this process or by one that ran before it on the GPU) downloads by DMA were seen to
 *       run at half rate for about 30 ms per GiB freed, uploads unaffected, whatever streams carry them.  No choice of
 *       streams changes that; *full_duplex_out (may be NULL) reports
 *       whether an upload and a download issued together overlapped when the call looked (1) or took turns (0).
 *       A process that wants the full-duplex rate allocates its long-lived buffers once and frees nothing large
 *       while it streams; one that reads 0 here can let the slots come back by a kernel instead
 *       (elixir_offload_set_evict_path below).  The two streams keep their directions: pass the first wherever this header takes
 *       h2d_stream and the second wherever it takes d2h_stream.  Allocates and frees 128 MiB of device and of pinned
 *       memory and waits for its probe copies (about 30 ms).  ELIXIR_TRACE_STREAMS=1 in the environment prints
 *       what was measured.  Streams of the caller's own making work with the pipeline as well, correctly but with no
 *       such guarantee.
 * No other call blocks the host.  h_block should be pinned (elixir_host_alloc) for
 * the copies to be asynchronous and at link speed.
 */
int elixir_host_alloc(void** h_out, size_t bytes);
int elixir_host_free(void* h_ptr);
int elixir_offload_register_slots(elixir_ctx* ctx, void* const* d_slots, int n_slots, size_t slot_bytes);
int elixir_offload_copy_streams(elixir_ctx* ctx, elixir_stream_t compute_stream, elixir_stream_t* h2d_out,
                                elixir_stream_t* d2h_out, int* full_duplex_out);
int elixir_chunk_prefetch(elixir_ctx* ctx, const void* h_block, size_t bytes, int* slot_out,
                          elixir_stream_t h2d_stream);
int elixir_chunk_wait_ready(elixir_ctx* ctx, int slot, elixir_stream_t compute_stream);
int elixir_chunk_evict(elixir_ctx* ctx, int slot, void* h_block, size_t bytes, elixir_stream_t compute_stream,
                       elixir_stream_t d2h_stream);

/*
 * How elixir_chunk_evict brings a slot back to its host block (no passage of the paper: a remedy for a state of the
 * HIP runtime).  ELIXIR_EVICT_DMA (the default): hipMemcpyAsync, the DMA engine.  ELIXIR_EVICT_KERNEL: a small kernel
 * on d2h_stream stores the slot into the pinned block over the link.  While downloads by DMA run at half rate
 * (elixir_offload_copy_streams reports that in *full_duplex_out; it follows the freeing of device memory and passes
 * with time) the kernel path lets the download run beside the upload at once.  The host block must then be pinned
 * memory that the device can address (elixir_host_alloc's is); for any other block, and for a slot or block that is
 * not 16-byte aligned, the call copies by DMA as before.  Takes effect from the next elixir_chunk_evict on; same bytes
 * either way.  ELIXIR_EINVAL for an unknown path.
 */
enum { ELIXIR_EVICT_DMA = 0, ELIXIR_EVICT_KERNEL = 1 };
int elixir_offload_set_evict_path(elixir_ctx* ctx, int path);

/*
 * The paper's own low-precision format, FP16 (Sec. 2 "Mixed Precision Training"), with dynamic loss scaling
 * (Micikevicius et al., "Mixed Precision Training", which the paper cites for its set-up; the paper gives no
 * rule of its own).  The *_lp entry points take the format as an argument and are otherwise the functions
 * above (which are the ELIXIR_LOWP_BF16 case).
 *   d_skip : DEVICE flag or NULL; when it is non-zero the update does nothing (master, moments and the
 *       low-precision copy keep their values): a step skipped because the scaled gradients overflowed.
 *   Loss-scale state, 16 bytes of DEVICE memory: scale S (the factor the caller multiplied the loss with),
 *       good_steps, skip, grad_scale.  elixir_loss_scale_init sets S.  elixir_loss_scale_update reads the
 *       norm of the SCALED gradients that elixir_chunk_grad_norm left in *d_norm_scaled (call it with
 *       max_norm <= 0) and, in a one-thread kernel: if the norm is Inf/NaN sets skip = 1, grad_scale = 0,
 *       S *= backoff_factor, good_steps = 0; otherwise skip = 0,
 *       grad_scale = min(1, max_norm / (norm/S + 1e-6)) / S  (max_norm <= 0: 1/S), good_steps += 1 and,
 *       when good_steps reaches growth_interval, S *= growth_factor and good_steps = 0.  Pass
 *       &state->grad_scale and &state->skip to the update; the new S is for the next iteration.
 */
typedef struct {
    float scale;
    int32_t good_steps;
    int32_t skip;
    float grad_scale;
} elixir_loss_scale_state;
int elixir_grad_reduce_into_chunk_lp(float* d_grad_chunk, int64_t offset, const uint16_t* d_grad_lowp, int lowp_format,
                                     int64_t n, float scale, int accumulate, elixir_stream_t stream);
/*
 * The reduction for many tensors in few launches: gradients arrive tensor by tensor and most tensors are small, so
 * one launch each leaves the GPU idle in between.  The tensors are cut into equal pieces plus tails, and pieces of
 * similar length share a launch as the rows of a 2-D grid (up to 336 rows; no host allocation; any number of tensors
 * at any addresses).  d_dst[i] points at the
 * tensor's place inside its fp32 gradient chunk (chunk base + offset, computed by the caller), d_grad_lowp[i] at its
 * n[i] low-precision gradients; all three tables are HOST arrays.  Destinations must not overlap.  Results are
 * bit-identical to n_tensors calls of elixir_grad_reduce_into_chunk_lp.
 */
int elixir_grad_reduce_multi_lp(int n_tensors, float* const* d_dst, const uint16_t* const* d_grad_lowp, const int64_t* n,
                                int lowp_format, float scale, int accumulate, elixir_stream_t stream);

/*
 * Several gradient arrays summed into the chunk in one pass.  With room for more than one set of low-precision
 * gradients (the next micro-batch's gradients while the previous ones are still there; on several GPUs the pieces
 * the other ranks sent for this rank's share of the chunk) the fp32 chunk need not be re-read and re-written once per
 * array:  for k < n, in this order,
 *   x = accumulate ? d_grad_chunk[offset+k] : 0;   for j = 0 .. n_sources-1:  x = fl32(x + fl32(scale * widen(d_grad_lowp[j][k])));
 *   d_grad_chunk[offset+k] = x
 * i.e. bit for bit what n_sources consecutive calls of elixir_grad_reduce_into_chunk_lp leave, at
 * 2*n_sources + 4 bytes per element instead of 10*n_sources - 4 (4 more on either side when accumulating).  d_grad_lowp is a HOST
 * array of n_sources device pointers; up to four arrays go into one pass, more are taken four at a time.
 * elixir_grad_reduce_sources_chunk_sumsq is elixir_grad_reduce_chunk_sumsq for several arrays (whole chunks, the sum
 * of squares of the final values left for elixir_chunk_grad_norm_finish).
 */
int elixir_grad_reduce_sources_lp(float* d_grad_chunk, int64_t offset, const uint16_t* const* d_grad_lowp, int n_sources,
                                  int lowp_format, int64_t n, float scale, int accumulate, elixir_stream_t stream);
int elixir_grad_reduce_sources_chunk_sumsq(elixir_ctx* ctx, int chunk_index, float* d_grad_chunk,
                                           const uint16_t* const* d_grad_lowp, int n_sources, int lowp_format,
                                           int64_t chunk_elems, int64_t valid_len, float scale, int accumulate,
                                           elixir_stream_t stream);
int elixir_chunk_adam_step_lp(float* d_master, float* d_exp_avg, float* d_exp_avg_sq, const float* d_grad_fp32,
                              const uint16_t* d_grad_lowp, uint16_t* d_param_lowp, int lowp_format, int64_t n,
                              const elixir_adam_hparams* hp, const float* d_grad_scale, const int32_t* d_skip,
                              elixir_stream_t stream);
int elixir_chunk_adam_step_multi_lp(int n_chunks, float* const* d_master, float* const* d_exp_avg,
                                    float* const* d_exp_avg_sq, const float* const* d_grad_fp32,
                                    const uint16_t* const* d_grad_lowp, uint16_t* const* d_param_lowp, int lowp_format,
                                    const int64_t* n, const elixir_adam_hparams* hp, const float* d_grad_scale,
                                    const int32_t* d_skip, elixir_stream_t stream);
int elixir_loss_scale_init(elixir_loss_scale_state* d_state, float init_scale, elixir_stream_t stream);
int elixir_loss_scale_update(elixir_loss_scale_state* d_state, const float* d_norm_scaled, float max_norm,
                             float growth_factor, float backoff_factor, int growth_interval, elixir_stream_t stream);

/*
 * CPU update of a host-resident chunk, the paper's own treatment of chunks kept in CPU memory: the
 * optimizer chunk never leaves the host, only low-precision gradients come down and low-precision
 * parameters go up (paper Sec. 2 "Memory Offloading"; CPU update velocity V_c in Sec. 5 and App. B).
 *   elixir_host_adam_step : the arithmetic of elixir_chunk_adam_step on HOST buffers, vectorised (AVX-512,
 *       AVX2 or scalar, chosen at run time) and spread over n_threads threads (<= 0: every core the process
 *       may run on).  Blocks until done.  grad_scale is a plain float (1 for no clipping).  Exactly one of
 *       h_grad_fp32 / h_grad_bf16 is non-NULL; h_param_bf16 may be NULL.
 *   elixir_host_adam_isa : "avx512", "avx2" or "scalar".
 *   elixir_copy_h2d_async / elixir_copy_d2h_async : asynchronous copies between pinned host memory and
 *       device memory on the caller's stream.  elixir_stream_synchronize : waits for a stream (the host
 *       must see the gradients before it updates, and the copy engines must be done with a host buffer
 *       before the CPU rewrites it).
 */
int elixir_host_adam_step(float* h_master, float* h_exp_avg, float* h_exp_avg_sq, const float* h_grad_fp32,
                          const uint16_t* h_grad_bf16, uint16_t* h_param_bf16, int64_t n,
                          const elixir_adam_hparams* hp, float grad_scale, int n_threads);
/* The same with the low-precision format as an argument (ELIXIR_LOWP_FP16: the paper's own format, IEEE binary16
 * gradients in, round-to-nearest-even binary16 parameters out, through the CPU's conversion instructions where it
 * has them); grad_scale carries 1/S under loss scaling.  elixir_host_adam_step is the ELIXIR_LOWP_BF16 case. */
int elixir_host_adam_step_lp(float* h_master, float* h_exp_avg, float* h_exp_avg_sq, const float* h_grad_fp32,
                             const uint16_t* h_grad_lowp, uint16_t* h_param_lowp, int lowp_format, int64_t n,
                             const elixir_adam_hparams* hp, float grad_scale, int n_threads);
int elixir_host_adam_step_tiled_lp(float* h_state, const float* h_grad_fp32, const uint16_t* h_grad_lowp, uint16_t* h_param_lowp,
                                   int lowp_format, int64_t n, const elixir_adam_hparams* hp, float grad_scale, int n_threads);
/* elixir_host_adam_step on a tiled optimizer chunk in host memory (the layout of elixir_state_tile). */
int elixir_host_adam_step_tiled(float* h_state, const float* h_grad_fp32, const uint16_t* h_grad_bf16, uint16_t* h_param_bf16,
                                int64_t n, const elixir_adam_hparams* hp, float grad_scale, int n_threads);
const char* elixir_host_adam_isa(void);
int elixir_copy_h2d_async(void* d_dst, const void* h_src, size_t bytes, elixir_stream_t stream);
int elixir_copy_d2h_async(void* h_dst, const void* d_src, size_t bytes, elixir_stream_t stream);
int elixir_stream_synchronize(elixir_stream_t stream);

/*
 * Offloading benefit model (paper Sec. 5.1, Eq. 1 and Eq. 2) and the placement rule built on it.  Host only.
 *   hw : aggregate bandwidths in BYTES per second (GPU to CPU, CPU to GPU) and aggregate update
 *        velocities in ELEMENTS per second (GPU, CPU) of the n_procs processes.
 *   elixir_offload_benefit : *I_out = I(n), the normalised time saved by one more rCache block;
 *        *J_out = J(n), the normalised time saved by moving one chunk and its update to the GPU.
 *        L_c, L_os: precision lengths in bytes (2 and 4); F_os: optimizer-state factor (3 for Adam).
 *   elixir_offload_plan : starts from min_blocks rCache blocks (the activation-checkpointing buffer
 *        size of App. A.3, at least 1) and all n_chunks chunks in CPU memory, and spends allowed_bytes
 *        (U_allowed, per GPU) on what has the larger benefit first: chunks moved to the GPU cost
 *        (L_c + L_os*F_os)*C/n_procs bytes each, rCache blocks L_c*C bytes each (at most n_chunks
 *        blocks: every chunk cached).  If allowed_bytes does not cover the mandatory blocks they are
 *        kept and nothing is moved.
 */
typedef struct {
    double b_g2c, b_c2g; /* bytes per second */
    double v_g, v_c;     /* elements per second */
} elixir_hw_profile;
int elixir_offload_benefit(int n_procs, int64_t chunk_elems, int L_c, int L_os, int F_os, const elixir_hw_profile* hw,
                           double* I_out, double* J_out);
int elixir_offload_plan(int n_procs, int64_t chunk_elems, int64_t n_chunks, int64_t min_blocks, int L_c, int L_os,
                        int F_os, const elixir_hw_profile* hw, double allowed_bytes, int64_t* n_blocks_out,
                        int64_t* n_gpu_chunks_out);

/*
 * rCache replacement simulation and chunk-size search (paper Sec. 3 "rCache": n_block equal blocks, Belady's
 * replacement from the known order of use; App. A.2: the chunk length that minimises the bytes replaced in
 * the rCache during one training step, found by simulating candidates).  Host only, integers.
 *   elixir_rcache_simulate : replays seq[0..len) (chunk ids, >= 0, dense) through n_blocks blocks, evicting
 *       the cached chunk whose next use lies farthest ahead (never used again first; ties: lowest id).
 *       *misses_out = accesses that found their chunk absent, *evictions_out = misses that displaced a chunk.
 *   elixir_chunk_size_search : for every candidate length plans the layout (policy, align_elems as for
 *       elixir_layout_plan), builds the access sequence of one step (parameters in order, then in reverse
 *       order; a parameter touches every chunk it spans; repeated accesses to the same chunk in a row
 *       count once), gives the cache floor(cache_bytes / (L_c * C)) blocks (at least 1) and records
 *       replaced_bytes_out[k] = evictions * L_c * C and, if padding_out is non-NULL, the padding elements.
 *       *best_out = index of the candidate with the fewest replaced bytes (ties: less padding, then the
 *       longer chunk).
 */
int elixir_rcache_simulate(const int64_t* seq, int64_t len, int64_t n_blocks, int64_t* misses_out,
                           int64_t* evictions_out);
int elixir_chunk_size_search(const int64_t* numel, int T, const int64_t* candidates, int n_cand, int policy,
                             int64_t align_elems, double cache_bytes, int L_c, int* best_out,
                             int64_t* replaced_bytes_out, int64_t* padding_out);

#ifdef __cplusplus
}
#endif
#endif /* ELIXIR_CHUNK_H */
