/*
 * nfd_attn.h - C ABI of the MI355X (gfx950) block-wise causal attention library.
 *
 * The operation is the attention of Next-Frame Diffusion (Sec. 3.1, paragraph
 * "Block-wise Causal Attention"): the token sequence is a run of frames of T
 * tokens each; a token attends to every token of its own frame and to every
 * token of all preceding frames, and to nothing in later frames.  The three
 * call forms of the paper map onto one entry point through (kv_frames,
 * q_frames):
 *   training / full sequence : q_frames == kv_frames            (Sec. 3.1)
 *   single-frame inference   : q_frames == 1 over cached frames (Appendix B, "KV Caching")
 *   speculative inference    : q_frames == N new frames over cached frames, block-causal
 *                              among themselves (Sec. 4.2; Appendix A listing)
 * The queries are always the LAST q_frames of the kv_frames frames held in k/v.
 *
 * All pointers named q, k, v, out, *_cache, *_new are DEVICE pointers on the
 * handle's device.  Tensors are dense and row-major.  Nothing here takes or
 * returns a torch type.  All work is enqueued on the caller's stream and the
 * calls do not synchronise with the host.  A handle may be used by one host
 * thread at a time; calls on one handle must be stream-ordered with respect
 * to each other (they share the handle's workspace).
 */
#ifndef NFD_ATTN_H
#define NFD_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct nfd_attn nfd_attn_t; /* opaque; owns only its workspace */

typedef enum { NFD_BF16 = 0, NFD_FP32 = 1 } nfd_dtype_t;

enum {
    NFD_OK = 0,
    NFD_ERR_NULL = -1,        /* a required pointer is NULL */
    NFD_ERR_SHAPE = -2,       /* a dimension < 1, or q_frames > kv_frames, or n_frames < 0 ... */
    NFD_ERR_UNSUPPORTED = -3, /* dtype / head width not built */
    NFD_ERR_CAPACITY = -4,    /* kv_frames > F, or frame_pos + n_frames > F */
    NFD_ERR_HIP = -5,         /* a HIP runtime call failed (text in nfd_last_error) */
    NFD_ERR_ALLOC = -6        /* host or device allocation failed */
};

/*
 * Create a handle for tensors of `dtype` on HIP device `device`.
 * workspace_bytes: device scratch owned by the handle, used for the partial
 * results of key-split launches (small query counts over a long cache); 0
 * selects a default (128 MiB).  A call whose ideal split does not fit the
 * workspace uses fewer splits; it never fails for that reason.
 * Allocates; not to be called under stream capture.
 * Errors: NFD_ERR_NULL (h), NFD_ERR_UNSUPPORTED (dtype), NFD_ERR_HIP, NFD_ERR_ALLOC.
 */
int nfd_attn_create(nfd_attn_t** h, nfd_dtype_t dtype, int device, size_t workspace_bytes);

/*
 * Block-wise causal attention forward (Sec. 3.1; cached and speculative forms:
 * Appendix B "KV Caching", Sec. 4.2 and the Appendix A listing).
 *
 *   P = kv_frames - q_frames                      past frames before the first query frame
 *   query row i in [0, q_frames*T), key j in [0, kv_frames*T)
 *   visible(i, j)  <=>  floor(j / T) <= P + floor(i / T)
 *   out[b,h,i,:] = softmax_j( scale * <q[b,h,i,:], k[b,h,j,:]> over visible j ) . v[b,h,j,:]
 *
 * q, out : [B, H, q_frames*T, D]
 * k, v   : [B, H, F*T, D]; F is the frame CAPACITY (head stride = F*T*D elements);
 *          only the first kv_frames*T rows of each head are read.  The K/V of the
 *          query frames themselves must already be in k, v (append first).
 * dtype of all four tensors is the handle's; bf16 computes on bf16 matrix cores
 * with fp32 accumulation and rounds the output to nearest-even; fp32 computes in fp32.
 * scale <= 0 selects 1/sqrt(D).  stream: a hipStream_t (NULL = default stream).
 * Supported: any B, H, T >= 1; D = 64 for bf16 on the matrix-core path (q, k, v, out 16-byte
 * aligned there), every other D <= 256 and all fp32 shapes on the general path.  The device current on the calling
 * thread must be the handle's device.
 * Ownership: the caller owns all four tensors; the library keeps no reference.
 * Errors (checked before any launch, in this order): NFD_ERR_NULL, NFD_ERR_SHAPE,
 * NFD_ERR_CAPACITY, NFD_ERR_UNSUPPORTED; NFD_ERR_HIP if a launch fails.
 */
int nfd_block_causal_attn_fwd(nfd_attn_t* h, const void* q, const void* k, const void* v, void* out,
                              int B, int H, int F, int T, int D, int kv_frames, int q_frames,
                              float scale, void* stream);

/*
 * One call for a cached step (Appendix B "KV Caching"; Sec. 4.2 for q_frames > 1): write the K/V of the q_frames
 * newest frames into the cache and attend.  Same result, bit for bit, in out and in the caches as
 *   nfd_kvcache_append(h, k_cache, v_cache, k_new, v_new, ..., frame_pos = kv_frames - q_frames, n_frames = q_frames)
 *   nfd_block_causal_attn_fwd(h, q, k_cache, v_cache, out, ..., kv_frames, q_frames)
 * but for bf16 with D = 64 in ONE launch: the attention reads the new frames' keys and values from k_new / v_new
 * where they are, and its workgroups copy them into the cache on the side (nothing in the launch reads the cache
 * rows that are being written).  Other dtypes / head widths, and calls with too few workgroups for the copy, run
 * the two launches.
 *   q, out : [B, H, q_frames*T, D]     k_new, v_new : [B, H, q_frames*T, D] (must not overlap the caches)
 *   k_cache, v_cache : [B, H, F*T, D]; frames [kv_frames - q_frames, kv_frames) of every head are overwritten
 * Errors as for nfd_block_causal_attn_fwd, plus NFD_ERR_NULL for k_new / v_new.
 */
int nfd_kvcache_append_attn_fwd(nfd_attn_t* h, const void* q, void* k_cache, void* v_cache, const void* k_new,
                                const void* v_new, void* out, int B, int H, int F, int T, int D, int kv_frames,
                                int q_frames, float scale, void* stream);

/*
 * nfd_block_causal_attn_fwd for callers that cannot allocate device memory and therefore cannot create a
 * handle: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  No handle;
 * the key-split partials, which the handle version keeps in its workspace, go to a fixed array of
 * NFD_NOALLOC_SCRATCH_BYTES inside the library's code object (each GPU the library runs on holds its own
 * copy until the process ends).  The call makes no hipMalloc / hipFree and no host heap allocation.
 *   dtype            : element type of q, k, v, out (as nfd_attn_create's)
 *   q, k, v, out ... : exactly as for nfd_block_causal_attn_fwd; runs on the device current on the calling thread
 *   err, err_len     : optional host buffer that receives the error text ("" on success); may be NULL / 0
 * The schedule is the one a handle with the default workspace uses, so the output is bit-identical to
 * nfd_block_causal_attn_fwd's.  A call whose partials would not fit the array (bf16, D = 64, key-split
 * launches only: B*H*q_frames*T*splits*136 bytes) is refused with NFD_ERR_ALLOC before anything is launched;
 * nothing is re-planned.  Calls that need no key split (training form, fp32, other head widths) use no scratch.
 * The array keeps the previous call's partials; nothing in it has to start at zero (every partial row a
 * launch reads, it has written before).  All calls on one GPU share the one array: calls that overlap in
 * time on the same GPU (two streams, two threads) race; order them on one stream.
 * The first call on a device looks up the array's device address and the device's properties: make it
 * outside stream capture.  Other errors as for nfd_block_causal_attn_fwd.
 */
#define NFD_NOALLOC_SCRATCH_BYTES ((size_t)32 << 20)
int nfd_block_causal_attn_fwd_noalloc(nfd_dtype_t dtype, const void* q, const void* k, const void* v, void* out, int B,
                                      int H, int F, int T, int D, int kv_frames, int q_frames, float scale, void* stream,
                                      char* err, size_t err_len);

/*
 * The same forward, additionally writing lse[b,h,i] = log sum_{visible j} exp(scale <q_i, k_j>)
 * (fp32, [B, H, q_frames*T]), which the backward call below consumes.  Arguments, support and
 * errors as for nfd_block_causal_attn_fwd; lse == NULL is NFD_ERR_NULL.
 */
int nfd_block_causal_attn_fwd_lse(nfd_attn_t* h, const void* q, const void* k, const void* v, void* out,
                                  float* lse, int B, int H, int F, int T, int D, int kv_frames, int q_frames,
                                  float scale, void* stream);

/*
 * Backward of the block-wise causal attention: the paper trains through this attention (Sec. 3.2
 * "Training"; mask of Sec. 3.1).  For the upstream gradient dout of out, with p_ij the softmax
 * weights of the visible keys:
 *   dv_j = sum_i p_ij dout_i      ds_ij = p_ij (<dout_i, v_j> - <dout_i, out_i>)
 *   dq_i = scale sum_j ds_ij k_j  dk_j = scale sum_i ds_ij q_i
 * q, out, dout, dq : [B, H, q_frames*T, D]     k, v, dk, dv : [B, H, F*T, D]     lse : [B, H, q_frames*T]
 * out and lse are the results of nfd_block_causal_attn_fwd_lse on the same q, k, v, scale.  Of dk and
 * dv only the first kv_frames*T rows of every head are written.  No atomics: results are
 * bit-reproducible.  Uses the handle's workspace (8 bytes per query row on the matrix-core path, 4 on the general one).
 * Supported: as the forward - bf16 with D = 64 on the matrix-core path (tensors 16-byte aligned there),
 * every other D <= 256 and all fp32 shapes on a general fp32-arithmetic path (one wavefront per row, not
 * tuned).
 * Errors, in this order: NFD_ERR_NULL, NFD_ERR_SHAPE, NFD_ERR_CAPACITY, NFD_ERR_UNSUPPORTED,
 * NFD_ERR_ALLOC (workspace too small), NFD_ERR_HIP.
 */
int nfd_block_causal_attn_bwd(nfd_attn_t* h, const void* q, const void* k, const void* v, const void* out,
                              const void* dout, const float* lse, void* dq, void* dk, void* dv, int B, int H,
                              int F, int T, int D, int kv_frames, int q_frames, float scale, void* stream);

/*
 * Write the K and V of n_frames new frames into the cache at frame frame_pos
 * (Appendix B, "KV Caching": K/V of a frame are computed once and reused by
 * every later denoising step and frame).
 * k_cache, v_cache : [B, H, F*T, D]      k_new, v_new : [B, H, n_frames*T, D]
 * Frames [frame_pos, frame_pos + n_frames) of every head are overwritten; this
 * is also how a rejected speculation is rolled back (Sec. 4.2): pass a smaller
 * kv_frames to the next forward and append from the last accepted frame.
 * n_frames == 0 is a no-op.  Errors: NFD_ERR_NULL, NFD_ERR_SHAPE,
 * NFD_ERR_CAPACITY (frame_pos + n_frames > F), NFD_ERR_UNSUPPORTED, NFD_ERR_HIP.
 */
int nfd_kvcache_append(nfd_attn_t* h, void* k_cache, void* v_cache, const void* k_new,
                       const void* v_new, int B, int H, int F, int T, int D, int frame_pos,
                       int n_frames, void* stream);

/*
 * 3D rotary position embedding of the queries and keys of n_frames new frames, fused with the
 * cache write: the step just before the attention call (Sec. 3.1, paragraph "3D Positional
 * Embedding": the head dimension of query and key tokens is separated into [n_T, n_H, n_W], a
 * rotary embedding is computed for each axis separately and the three are concatenated along the
 * last dimension; Appendix B "KV Caching" for the cache).
 *
 *   token tok of new frame f sits at (t, y, x) = (t_offset + frame_pos + f, tok / grid_w, tok % grid_w)
 *   features [0, n_t) follow t, [n_t, n_t + n_h) follow y, [n_t + n_h, D) follow x
 *   inside a section of width n, pair (2i, 2i+1) at position p turns by p * theta^(-2i/n):
 *       (a, b) -> (a cos - b sin, a sin + b cos)
 *
 * q, q_out       : [B, H, n_frames*T, D]; q_out receives the rotated queries and may be q itself
 * k_new, v_new   : [B, H, n_frames*T, D]
 * k_cache, v_cache : [B, H, F*T, D]; frames [frame_pos, frame_pos + n_frames) of every head receive the
 *                  rotated keys and the unchanged values
 * T must equal grid_h * grid_w; n_t, n_h, n_w are even, >= 0 and sum to D; theta > 0 (theta <= 0
 * selects 10000); t_offset shifts the temporal positions (a sliding context window).
 * Angles are formed in fp64, the rotation in fp32, the result rounded to the handle's dtype (RNE).
 * n_frames == 0 is a no-op.  Errors, in this order: NFD_ERR_NULL, NFD_ERR_SHAPE (also a grid or
 * section mismatch), NFD_ERR_CAPACITY, NFD_ERR_UNSUPPORTED (D > 256), NFD_ERR_HIP.
 * Ownership as for the other calls: the library keeps no reference.
 */
int nfd_rope_kvcache_append(nfd_attn_t* h, const void* q, void* q_out, void* k_cache, void* v_cache,
                            const void* k_new, const void* v_new, int B, int H, int F, int T, int D,
                            int frame_pos, int n_frames, int t_offset, int grid_h, int grid_w, int n_t,
                            int n_h, int n_w, float theta, void* stream);

/* The argument checks of nfd_rope_kvcache_append that do not need pointers, same order and codes
 * (host only, no HIP call). */
int nfd_rope_check_args(nfd_dtype_t dtype, int B, int H, int F, int T, int D, int frame_pos, int n_frames,
                        int grid_h, int grid_w, int n_t, int n_h, int n_w);

/*
 * Slide the context window (Sec. 5 "Limitations": the context is limited to a fixed number of frames):
 * drop the oldest n_drop of the kv_frames cached frames of every head by moving frames
 * [n_drop, kv_frames) to [0, kv_frames - n_drop).  k_cache, v_cache : [B, H, F*T, D].  Overlapping
 * moves go through the handle's workspace when it is large enough, otherwise in runs of n_drop frames.
 * The temporal positions of the remaining frames do not change: pass t_offset += n_drop to the next
 * rotary-embedding call.  n_drop == 0 is a no-op.
 * Errors: NFD_ERR_NULL, NFD_ERR_SHAPE (also n_drop > kv_frames), NFD_ERR_CAPACITY (kv_frames > F), NFD_ERR_HIP.
 */
int nfd_kvcache_shift(nfd_attn_t* h, void* k_cache, void* v_cache, int B, int H, int F, int T, int D,
                      int kv_frames, int n_drop, void* stream);

/*
 * Bookkeeping of speculative sampling (Sec. 4.2 "Speculative Sampling"; Appendix A, "Detailed Algorithm of
 * Speculative Sampling"): every model call generates n_spec frames under the CURRENT action repeated;
 * afterwards the true actions of those frames are compared with it, the leading frames whose action
 * matches are kept, the rest is discarded and generation resumes after the last verified frame.  Host
 * only: no GPU, no HIP call, no allocation; the struct is plain data owned by the caller.
 *
 * Reading of the listing's `first_change_idx + 1`: the number of kept frames is the length of the run of
 * the current action at the start of the chunk (at least 1: the first frame is generated under its own
 * action).  Discarding needs no device work: the next call passes a smaller kv_frames and its append
 * overwrites the rejected frames' K/V.
 */
typedef struct nfd_spec {
    int capacity; /* F: frames the cache can hold */
    int window;   /* frames of verified context kept; window + n_spec <= capacity */
    int n_spec;   /* N: frames generated per model call */
    int total;    /* frames of the whole video, prompt included */
    int done;     /* frames verified so far, prompt included (the listing's i) */
    int cached;   /* verified frames now in the cache */
    int t_offset; /* absolute index of the frame in cache slot 0 */
} nfd_spec_t;

typedef struct nfd_spec_step {
    int n_drop;    /* oldest frames to evict first: nfd_kvcache_shift(kv_frames = frame_pos + n_drop, n_drop) */
    int frame_pos; /* cache frame where the new frames' K/V are appended */
    int n_frames;  /* frames this call generates: min(n_spec, total - done) */
    int kv_frames; /* arguments of the attention call: frame_pos + n_frames ... */
    int q_frames;  /* ... and n_frames */
    int t_offset;  /* temporal offset for the rotary embedding, after the eviction */
} nfd_spec_step_t;

/* n_prompt given frames are already in the cache.  Errors: NFD_ERR_NULL, NFD_ERR_SHAPE,
 * NFD_ERR_CAPACITY (window + n_spec > capacity or n_prompt > capacity). */
int nfd_spec_init(nfd_spec_t* s, int capacity, int window, int n_spec, int n_prompt, int total);
/* Describe the next model call and apply its eviction to the bookkeeping.  Returns 1 if a call is
 * due, 0 when all frames are done, < 0 on NULL. */
int nfd_spec_next(nfd_spec_t* s, nfd_spec_step_t* step);
/* After the call: actions is the host array [total, action_dim] of the true actions; *accepted
 * receives the number of frames kept (1 .. step->n_frames).  Errors: NFD_ERR_NULL, NFD_ERR_SHAPE. */
int nfd_spec_accept(nfd_spec_t* s, const nfd_spec_step_t* step, const int32_t* actions, int action_dim,
                    int* accepted);

/* Free the handle and its workspace.  NULL is accepted. */
int nfd_attn_destroy(nfd_attn_t* h);

/* Text of the last error on this handle ("" if none); valid until the next call on it. */
const char* nfd_last_error(const nfd_attn_t* h);

/* ---- host-only helpers: no GPU needed, no HIP call made ------------------------------- */

/* The argument checks of nfd_block_causal_attn_fwd that do not need pointers
 * (shape, capacity, support), in the same order and with the same codes. */
int nfd_attn_check_args(nfd_dtype_t dtype, int B, int H, int F, int T, int D, int kv_frames,
                        int q_frames);

/* The tile schedule the forward would launch (Sec. 3.1: skipping the tiles of
 * future frames IS the ~50 % saving the paper states). */
typedef struct nfd_attn_plan {
    int kernel;          /* 0 = general (fp32 / any D), 1 = bf16 matrix-core D=64 */
    int block_m;         /* query rows per workgroup, at most: the 32-row blocks of a head are dealt evenly to its
                            n_q_tiles tiles (tile i owns floor(blocks / n_q_tiles) blocks, the first blocks mod n_q_tiles
                            tiles one more) */
    int block_n;         /* keys per inner tile */
    int n_q_tiles;       /* query tiles per (b, h) */
    int n_splits;        /* key splits per query tile (1 = no combine pass) */
    int n_workgroups;    /* total workgroups of the main launch */
    int64_t key_tiles_visited; /* sum over workgroups of key tiles actually visited */
    int64_t key_tiles_dense;   /* the same count if no future tile were skipped */
    size_t workspace_bytes;    /* scratch the split launch needs (0 if n_splits == 1) */
} nfd_attn_plan_t;

/* num_cus <= 0 selects 256; workspace_limit == 0 selects the default workspace. */
int nfd_attn_plan(nfd_dtype_t dtype, int B, int H, int F, int T, int D, int kv_frames,
                  int q_frames, int num_cus, size_t workspace_limit, nfd_attn_plan_t* plan);

/*
 * 8-bit KV cache.  Appendix B's cache held as OCP E4M3 codes (1 sign, 4 exponent, 3 mantissa bits, bias 7,
 * largest value 448): the post-training quantisation that Sec. 6 names as a further acceleration and leaves
 * out.  The paper fixes no format; this one keeps the attention arithmetic unchanged: one scale per
 * (batch, head) and tensor, supplied by the caller; code = E4M3(x / scale), nearest-even, saturating at
 * +-448, x / scale formed as x * (1 / scale) in fp32; value read = code * scale.  The attention kernel
 * widens the codes to bf16 (exact) on their way into the matrix cores and applies the scales to the softmax
 * scale (K) and to the final result (V).
 * Layouts (device memory, 16-byte aligned, owned by the caller):
 *   k8  : [B, H, Spad, D] codes          v8t : [B, H, D, Spad] codes (feature-major)
 *   Spad = F * T rounded up to a multiple of 64;  nfd_fp8_cache_bytes returns the size of EACH cache.
 *   Inside every aligned group of 16 keys of a v8t row the order is permuted: key q = 4a + b of the group
 *   (a = 0..3, b = 0..3) sits at byte 8 * ((a & 1) ^ s) + 4 * (a >> 1) + b, s = bit 4 of the feature index.
 *   Both caches are written by nfd_kvcache_append_fp8 and moved by nfd_kvcache_shift_fp8 only.
 *   k_scale, v_scale : [B, H] fp32, positive.
 * Codes outside the first kv_frames * T keys are never used, whatever they are.  Supported: bf16 handle, D = 64.
 */
int nfd_fp8_cache_bytes(int B, int H, int F, int T, int D, size_t* bytes);

/* Quantise n_frames new frames (k_new, v_new: [B, H, n_frames*T, D] bf16) into frames frame_pos.. of the 8-bit
 * caches.  Errors as nfd_kvcache_append, plus NFD_ERR_UNSUPPORTED for fp32 handles, D != 64 or misaligned
 * tensors. */
int nfd_kvcache_append_fp8(nfd_attn_t* h, void* k8, void* v8t, const float* k_scale, const float* v_scale,
                           const void* k_new, const void* v_new, int B, int H, int F, int T, int D, int frame_pos,
                           int n_frames, void* stream);

/* nfd_rope_kvcache_append writing the 8-bit caches: q is rotated into q_out; the rotated key, rounded to bf16
 * exactly as for a bf16 cache, and the value are quantised as by nfd_kvcache_append_fp8.  The codes equal those of
 * nfd_rope_kvcache_append into a bf16 buffer followed by nfd_kvcache_append_fp8.  Errors as for
 * nfd_rope_kvcache_append, plus NFD_ERR_NULL for the scales and NFD_ERR_UNSUPPORTED for fp32 handles, D != 64 or
 * tensors that are not 16-byte aligned. */
int nfd_rope_kvcache_append_fp8(nfd_attn_t* h, const void* q, void* q_out, void* k8, void* v8t, const float* k_scale,
                                const float* v_scale, const void* k_new, const void* v_new, int B, int H, int F,
                                int T, int D, int frame_pos, int n_frames, int t_offset, int grid_h, int grid_w,
                                int n_t, int n_h, int n_w, float theta, void* stream);

/* nfd_kvcache_shift for the 8-bit caches: frames n_drop .. kv_frames-1 move to frames 0 .. ; same strategies
 * and errors (NFD_ERR_UNSUPPORTED for D != 64).  When T is a multiple of 16 whole key groups move (16-byte
 * vectors); otherwise V moves key by key through the handle's workspace, which must hold at least one feature
 * row of the kept keys ((kv_frames - n_drop) * T bytes), else NFD_ERR_ALLOC before anything is launched. */
int nfd_kvcache_shift_fp8(nfd_attn_t* h, void* k8, void* v8t, int B, int H, int F, int T, int D, int kv_frames,
                          int n_drop, void* stream);

/* nfd_block_causal_attn_fwd with K and V read from the 8-bit caches; q and out are bf16.  Same schedule,
 * key splits and errors; NFD_ERR_UNSUPPORTED for fp32 handles or D != 64. */
int nfd_block_causal_attn_fwd_fp8kv(nfd_attn_t* h, const void* q, const void* k8, const void* v8t,
                                    const float* k_scale, const float* v_scale, void* out, int B, int H, int F,
                                    int T, int D, int kv_frames, int q_frames, float scale, void* stream);

/* Which (head, query tile, key split) workgroup `block` of the matrix-core forward launch works on: the
 * same function the kernel evaluates, exposed so that the schedule can be checked without a GPU (every item
 * exactly once over blocks 0 .. n_workgroups-1).  group_q_tiles: the ordering used when K/V exceed the
 * last-level cache.  Errors: NFD_ERR_NULL, NFD_ERR_SHAPE (also a block past the launch). */
int nfd_attn_work_item(int BH, int n_q_tiles, int n_splits, int group_q_tiles, unsigned block, int* bh, int* q_tile,
                       int* split);

/* Query rows [first_row, first_row + n_rows) of query tile q_tile when a head's `rows` query rows are cut into
 * n_q_tiles tiles (the plan's count) for the matrix-core forward: the same function the kernel evaluates.  The 32-row
 * blocks are dealt evenly (tile sizes differ by at most 32 rows); the tiles are disjoint and cover all rows.
 * Errors: NFD_ERR_NULL, NFD_ERR_SHAPE, NFD_ERR_UNSUPPORTED (rows beyond the 2^30 of the attention calls). */
int nfd_attn_q_tile_rows(int rows, int n_q_tiles, int q_tile, int* first_row, int* n_rows);

/* Visible (query, key) pairs per (b, h): T^2 (q_frames P + q_frames (q_frames + 1) / 2). */
int64_t nfd_attn_visible_pairs(int T, int kv_frames, int q_frames);

#ifdef __cplusplus
}
#endif
#endif /* NFD_ATTN_H */
