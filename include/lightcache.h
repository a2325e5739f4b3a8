/*
 * lightcache.h - C ABI of the MI355X (gfx950) library for the cache-hit denoising step of a
 * DeepCache-style video UNet with asynchronous cache swapping and feature chunking.
 *
 * Method references are to the LightCache paper (arXiv 2510.05367):
 *   [FC]   "Feature Calculation" paragraph, eq. U_i = Concat(D_i, U_{i+1})
 *   [AS]   "Asynchronous Swapping" section (DeepCache cache equation, refresh interval n,
 *          cached features kept on the CPU and brought back in the background)
 *   [CHK]  "Feature chunk and Sliced Decoding" section, eq. Chunk(F)
 *
 * Conventions
 *   - Every pointer argument is annotated [device] or [host]. Device pointers must be valid on
 *     the GPU that was current when lc_create() was called.
 *   - Public tensors use the paper's order [B, F, C, H, W] ([CHK]); B*F is written N. Elements
 *     are lc_config.dtype (float, or bf16 stored as uint16).
 *   - Every function returns lc_status; on error no output argument is written and a message is
 *     available from lc_last_error(). Nothing aborts or throws across this boundary.
 *   - Step and swap calls only *enqueue* work (on the compute stream and the side stream given
 *     to lc_create) and return; lc_sync() drains both. Ordering between a step and a swap that
 *     touch the same device slot is enforced inside the library with events.
 *   - After lc_set_workspace() no call allocates or frees device memory.
 *   - Lifetime of arguments: a [device] tensor passed to a step, an operator, lc_cache_write or
 *     lc_cache_read is read or written by work that is only enqueued when the call returns. It must stay
 *     valid, and must not be handed to other work on another stream, until lc_sync() has returned or an event
 *     recorded on the compute stream after the call has completed. With a caching allocator this means:
 *     allocate such tensors on the compute stream or keep a reference until then.
 *   - lc_cache_peek / lc_cache_dev_peek return raw pointers with no ordering against a swap or step in
 *     flight: call lc_sync() first.
 */
#ifndef LIGHTCACHE_H
#define LIGHTCACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lc_ctx lc_ctx; /* opaque; owned by the library */

typedef enum {
  LC_OK = 0,
  LC_ERR_ARG = 1,   /* NULL pointer, slot out of range, negative chunk, bad enum */
  LC_ERR_SHAPE = 2, /* configuration the kernels do not support */
  LC_ERR_STATE = 3, /* call order: empty slot, weights / workspace not set */
  LC_ERR_NOMEM = 4, /* workspace too small, host allocation failed */
  LC_ERR_HIP = 5    /* a HIP runtime call failed */
} lc_status;

typedef enum { LC_F32 = 0, LC_BF16 = 1 } lc_dtype;

/* Shape of the shallow stage. Requirements (else LC_ERR_SHAPE): all > 0; H, W even;
 * C, C_deep multiples of 64; C, C_deep and C + C_deep divisible by groups; heads * head_dim == C;
 * head_dim a multiple of 8 and <= 64; C_lat <= 16; n_res <= LC_MAX_RES; 1 <= dev_slots <= 8;
 * 0 <= host_slots <= 64. */
typedef struct lc_config {
  int32_t B, F, H, W;      /* batch (2 with classifier-free guidance), frames, latent size */
  int32_t C_lat, C, C_deep; /* latent channels, stage channels, deep-feature channels (at H/2 x W/2) */
  int32_t groups, n_res;   /* GroupNorm groups; residual blocks on the down side */
  int32_t heads, head_dim;
  int32_t dtype;           /* lc_dtype: storage type of activations, weights, x, eps, cache */
  float gn_eps;
  int32_t host_slots;      /* entries of the pinned host cache bank */
  int32_t dev_slots;       /* device buffers for deep features (2 = double buffered) */
} lc_config;

#define LC_MAX_RES 4

/* Weights, all [device], element type lc_config.dtype, PyTorch layouts:
 * conv w [Cout, Cin, 3, 3], linear w [Cout, Cin], vectors [C]. The library makes packed private
 * copies during lc_load_weights(); the caller's buffers may be freed afterwards. */
typedef struct lc_gnconv_w { const void *gn_g, *gn_b, *w, *b; } lc_gnconv_w;
typedef struct lc_attn_w { const void *gn_g, *gn_b, *wq, *wk, *wv, *wo, *bo; } lc_attn_w;
typedef struct lc_weights {
  const void *conv_in_w, *conv_in_b; /* C_lat -> C */
  lc_gnconv_w res[LC_MAX_RES];       /* GN(C) -> SiLU -> conv C -> C, + identity */
  lc_attn_w sattn, tattn;            /* spatial / temporal self-attention blocks */
  const void *down_w, *down_b;       /* deep stand-in: stride-2 conv C -> C_deep */
  lc_gnconv_w dres;                  /* deep stand-in: residual block at C_deep */
  lc_gnconv_w up;                    /* GN(C + C_deep) -> SiLU -> conv (C + C_deep) -> C */
  lc_gnconv_w out;                   /* GN(C) -> SiLU -> conv C -> C_lat */
} lc_weights;

/* Counters since lc_create (or the last lc_reset_stats). Times are GPU times from events. */
typedef struct lc_stats {
  int64_t full_steps, cached_steps, swaps_out, swaps_in;
  int64_t bytes_out, bytes_in;      /* bytes moved device->host / host->device */
  double ms_out, ms_in;             /* summed copy durations (completed, timed copies only) */
  int64_t timed_out, timed_in;      /* copies ms_out / ms_in cover (a copy issued while all 256 timing event
                                       pairs were still in flight is counted in swaps_* but not timed) */
  size_t workspace_bytes;           /* arena bytes in use for the current chunk setting */
  size_t weight_bytes;              /* device bytes of the packed private weight copies */
  size_t host_bank_bytes;           /* pinned host bytes */
} lc_stats;

/* Kernel families for per-kernel timing (lc_set_profiling / lc_get_profile). */
enum {
  LC_K_CONV_IN = 0, LC_K_GN_STATS, LC_K_GN_FINAL, LC_K_GN_APPLY, LC_K_CONV_RES, LC_K_QKV,
  LC_K_SATTN, LC_K_TATTN, LC_K_PROJ, LC_K_CAT_APPLY, LC_K_CONV_UP, LC_K_CONV_OUT, LC_K_DEEP,
  LC_K_COUNT
};
typedef struct lc_profile {
  double ms[LC_K_COUNT];
  int64_t launches[LC_K_COUNT];
  int64_t dropped; /* launches of bracketed families that ran untimed because the bracket pool was full */
} lc_profile;

/* ---- host-only helpers (no GPU needed) ------------------------------------------------- */

/* Validates a configuration against the requirements above. cfg: [host]. */
lc_status lc_check_config(const lc_config* cfg);

/* Bytes of one cache entry (deep feature [N, C_deep, H/2, W/2]); 0 if cfg is invalid. */
size_t lc_cache_entry_bytes(const lc_config* cfg);

/* Footprint model: arena bytes lc_set_workspace() needs for the given chunk setting (persistent
 * skip feature + dev_slots cache entries + chunk-sized scratch). frame_chunk / token_chunk as in
 * lc_set_chunk(); with a chunk set, the chunk scratch is counted twice (see lc_set_lanes()).
 * Returns 0 if cfg is invalid or a chunk is negative. */
size_t lc_workspace_bytes(const lc_config* cfg, int frame_chunk, int token_chunk);

/* The same with a spatial chunk (lc_set_spatial_chunk) of eta x omega blocks. 0 if the factors do not divide H, W. */
size_t lc_workspace_bytes_spatial(const lc_config* cfg, int frame_chunk, int token_chunk, int eta, int omega);

/* Message of the most recent error on this ctx (ctx == NULL: of the calling thread's last
 * ctx-less call). Never NULL; valid until the next call on the same ctx / thread. */
const char* lc_last_error(const lc_ctx* ctx);

/* ---- lifetime -------------------------------------------------------------------------- */

/* Creates a context on the current device. compute_stream / side_stream: hipStream_t handles
 * owned by the caller (e.g. torch.cuda.Stream().cuda_stream), default priority, distinct, must
 * outlive the ctx. Allocates the pinned host bank (host_slots entries). */
lc_status lc_create(const lc_config* cfg, void* compute_stream, void* side_stream, lc_ctx** out);

/* Drains both streams and frees everything the library owns. NULL is a no-op. A pointer that lc_create did
 * not return, or that has been destroyed before, is not dereferenced: LC_ERR_ARG. */
lc_status lc_destroy(lc_ctx* ctx);

/* Test hook for the error path of lc_create: the nth pinned allocation (1-based) that lc_create calls on this
 * host thread make from now on fails as if the host were out of memory, once (0 = off). lc_create then
 * returns LC_ERR_NOMEM and leaves nothing allocated. */
lc_status lc_test_fail_host_alloc(int nth);

/* Packs the weights into private device copies (allocates; synchronises the compute stream). */
lc_status lc_load_weights(lc_ctx* ctx, const lc_weights* w /* [host] struct of [device] ptrs */);

/* Hands the library a caller-owned arena ([device], 256-byte aligned, >= lc_workspace_bytes for
 * the current chunk setting, else LC_ERR_NOMEM). Cache slots become empty. The arena must stay
 * valid until lc_destroy or the next lc_set_workspace. */
lc_status lc_set_workspace(lc_ctx* ctx, void* arena, size_t bytes);

/* ---- the method ------------------------------------------------------------------------ */

/* Feature chunk ([CHK]). frame_chunk = frames of the flattened B*F axis processed per pass by
 * the per-frame operators; token_chunk = spatial positions per pass of temporal attention and
 * query tokens per pass of spatial attention. 0 = unchunked; values above the axis length clamp;
 * a chunk that does not divide the axis gives a short last pass. If token_chunk == 0 and
 * frame_chunk > 0, temporal attention uses ceil(frame_chunk * H*W / (B*F)) positions per pass
 * (as many rows as a frame chunk). Chunking never changes results (each output is reduced in the
 * same order). LC_ERR_NOMEM if a workspace is set and is too small for the new setting. */
lc_status lc_set_chunk(lc_ctx* ctx, int frame_chunk, int token_chunk);

/* Spatial feature chunk ([CHK], eq. Chunk(F): F_i of size H/eta x W/omega). Every operator of the shallow branch
 * then runs block by block over the eta x omega spatial blocks of each frame (inside the frame chunks above): the
 * 3x3 convolutions and conv_in / conv_out compute a block's pixels with the one-pixel halo read from the
 * neighbouring blocks of their input; GroupNorm statistics are split sums per block, folded once all blocks of the
 * producing operator are done (two passes); the projections take a block's positions; spatial attention takes a
 * block's queries against the keys and values of the whole frame; temporal attention takes a block's positions
 * (the blocks replace token_chunk). Results are identical bit for bit to the unchunked step: a block is made of
 * whole tiles of every kernel, which is what restricts the factors: eta must divide H with H/eta a multiple of 8,
 * omega must divide W with W/omega a multiple of 32, eta * omega <= 64, C in {64, 128} or 320 with bf16, C_lat <= 7;
 * otherwise LC_ERR_SHAPE. (1, 1) = off, the default. LC_ERR_ARG for factors below 1; LC_ERR_NOMEM if a workspace
 * is set and is too small (the temporal pass then works on N * H/eta * W/omega rows: lc_workspace_bytes_spatial).
 * The deep stand-in of the normal step is not chunked spatially. */
lc_status lc_set_spatial_chunk(lc_ctx* ctx, int eta, int omega);

/* Chunk overlap. The chunks of a step ([CHK]) depend on each other only where the method joins
 * them (before temporal attention, before the up branch, at the end), so a chunked step issues
 * alternate chunks on two streams - the compute stream and one of the library's own, forked from
 * and joined back into the compute stream inside every step, so the caller still orders work
 * against the compute stream alone - each with its own chunk scratch (lc_workspace_bytes counts the
 * second copy whenever a chunk is set). lanes = 1 keeps everything on the compute stream; 2 is the
 * default. Results are identical bit for bit. While per-kernel profiling is on (lc_set_profiling)
 * steps run on one lane, so that a timed kernel has the device to itself. LC_ERR_ARG unless
 * lanes is 1 or 2. */
lc_status lc_set_lanes(lc_ctx* ctx, int lanes);

/* Kernel choice of the 3x3 convolutions of the shallow branch (residual blocks, up conv; the operations of
 * [FC] and of the residual blocks are the same either way). A bf16 stage whose widths allow it
 * (C % 160 == 0) runs them in a kernel whose wavefronts are specialised (loaders / contracting); general = 1
 * forces the general kernel, which every other stage uses anyway. The two accumulate the same products in
 * the same order: results are identical bit for bit (this switch exists so that a test can say so).
 * Default 0. LC_ERR_ARG unless general is 0 or 1. */
lc_status lc_set_conv_general(lc_ctx* ctx, int general);

/* Normal step ([AS]: the steps t = 0, n, 2n, ...): shallow down branch, deep stand-in, shallow
 * up branch on Concat(skip, deep) ([FC]); the deep feature is left in device slot dev_slot.
 * x [device, B,F,C_lat,H,W] -> eps [device, same shape]. Both must stay valid until the compute
 * stream has been synchronised. */
lc_status lc_full_step(lc_ctx* ctx, const void* x, void* eps, int dev_slot);

/* Cache step ([AS]): only the shallow branch is recomputed; the deep feature is read from device
 * slot dev_slot (filled by lc_full_step, lc_swap_in or lc_cache_write; LC_ERR_STATE if empty).
 * If a swap-in into that slot is in flight the step waits for it on the GPU, just before the up
 * branch. */
lc_status lc_cached_step(lc_ctx* ctx, const void* x, void* eps, int dev_slot);

/* For callers that cannot allocate device memory and have none to hand over as a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc. The same cache step as lc_cached_step,
 * with the library's own static device array (LC_STATIC_SCRATCH_BYTES per GPU, held from library load until the
 * process ends) as its arena, so neither lc_set_workspace nor a filled device slot is needed, and the call
 * itself allocates nothing (no hipMalloc / hipFree, no allocating library routine).
 * x [device, B,F,C_lat,H,W] -> eps [device, same shape]; deep [device, N, C_deep, H/2, W/2], public layout as
 * in lc_cache_write: the deep feature to concatenate ([FC]); it is copied into the scratch in the library's
 * layout first. All three stay valid until the compute stream has been synchronised.
 * LC_ERR_NOMEM if lc_workspace_bytes(cfg, current chunk setting) > LC_STATIC_SCRATCH_BYTES (a smaller chunk may
 * fit; the AnimateDiff-sized stages do not). LC_ERR_STATE without weights. The context's own workspace,
 * device slots and cache bank are not touched. Every call on a GPU shares that GPU's array, whichever context
 * it comes from, and finds the last call's contents there (nothing in it needs clearing: every kernel writes
 * what it later reads): calls are safe one after the other on one compute stream; calls that overlap on one
 * GPU (two contexts on different streams, two host threads) race. */
#define LC_STATIC_SCRATCH_BYTES (64u << 20)
lc_status lc_cached_step_static(lc_ctx* ctx, const void* x, const void* deep, void* eps);
size_t lc_static_scratch_bytes(void); /* LC_STATIC_SCRATCH_BYTES as the library was built */

/* Asynchronous cache swapping ([AS]). Both enqueue one copy on the side stream and return.
 * swap_out: device slot -> host bank entry, after the work that produced the slot.
 * swap_in : host bank entry -> device slot, after the last enqueued step that reads the slot.
 * LC_ERR_STATE on an empty source. */
lc_status lc_swap_out(lc_ctx* ctx, int dev_slot, int host_slot);
lc_status lc_swap_in(lc_ctx* ctx, int host_slot, int dev_slot);

/* Blocks the host until both streams are idle. */
lc_status lc_sync(lc_ctx* ctx);

/* ---- cache access for tests and for injecting a deep feature ---------------------------- */

/* Fills device slot from / copies it to a tensor in public layout [N, C_deep, H/2, W/2]
 * ([device], cfg dtype), on the compute stream. The slot's internal layout is private. */
lc_status lc_cache_write(lc_ctx* ctx, int dev_slot, const void* deep);
lc_status lc_cache_read(lc_ctx* ctx, int dev_slot, void* deep);

/* Raw views for byte-exact checks (no copy, no sync): *ptr [host] for a bank entry, [device]
 * for a slot; *bytes = lc_cache_entry_bytes. */
lc_status lc_cache_peek(lc_ctx* ctx, int host_slot, const void** ptr, size_t* bytes);
lc_status lc_cache_dev_peek(lc_ctx* ctx, int dev_slot, const void** ptr, size_t* bytes);

/* ---- measurement ------------------------------------------------------------------------ */

lc_status lc_get_stats(lc_ctx* ctx, lc_stats* out /* [host] */); /* synchronises the side stream */
lc_status lc_reset_stats(lc_ctx* ctx);

/* mask: bit k set = bracket every launch of kernel family k (LC_K_*) with events on the compute
 * stream. lc_get_profile() synchronises, sums the brackets into out and clears them. At most
 * 4096 brackets are kept between two lc_get_profile calls; further launches are not timed and are
 * counted in lc_profile.dropped. */
lc_status lc_set_profiling(lc_ctx* ctx, uint32_t mask);
lc_status lc_get_profile(lc_ctx* ctx, lc_profile* out /* [host] */);

/* ---- single operators (the same kernels the steps launch; used by the parity tests and the
 *      benchmark). Activations are in the library's internal channels-last layout
 *      [rows, channels] with rows = frame-major pixels; all pointers [device].
 *      Element types: tensors of the residual stream (h, u, d0 below: what every block adds into)
 *      are always float: with bf16 storage that stream is kept in fp32 and only MFMA operands are
 *      rounded. Operand tensors (qkv, attention outputs, cache entries) and the public x / eps
 *      have the cfg dtype. GroupNorm (+ SiLU), the 2x upsampling and the skip-concat are applied
 *      inside the loaders of the kernels that consume them, so they appear here only as part of
 *      the operator they feed. Each call enqueues on the compute stream. `frames` counts frames of
 *      H x W pixels (H/2 x W/2 where stated) and is at most B*F. ------------------------------- */

typedef enum {
  LC_L_RES0 = 0, /* .. LC_L_RES0 + n_res - 1 */
  LC_L_SATTN = 8, LC_L_TATTN = 9, LC_L_DRES = 10
} lc_layer;

/* h[frames*H*W, C] (float) = conv_in(x[frames, C_lat, H, W]). */
lc_status lc_op_conv_in(lc_ctx* ctx, const void* x, void* h, int frames);
/* Residual block body, y = x + conv3x3(SiLU(GroupNorm(x))), x float, y != x.
 * LC_L_RESi: [frames*H*W, C], y float. LC_L_DRES: [frames*(H/2)*(W/2), C_deep], y cfg dtype (it
 * writes a cache entry). */
lc_status lc_op_res_block(lc_ctx* ctx, int layer, const void* x, void* y, int frames);
/* qkv[frames*H*W, 3C] (cfg dtype) = GroupNorm(x)[rows, C] [Wq;Wk;Wv]^T of LC_L_SATTN / LC_L_TATTN,
 * x float, statistics per frame. For LC_L_SATTN the q third is stored multiplied by
 * log2(e)/sqrt(head_dim), scaled before it is rounded: the form lc_op_spatial_attention takes with
 * q_prescaled = 1 and the steps use between the two kernels. */
lc_status lc_op_qkv(lc_ctx* ctx, int layer, const void* x, void* qkv, int frames);
/* Whole attention blocks, in place on the float rows h (the sequence of launches a step issues, on the chunk
 * scratch): h += proj(Attn(qkv(GroupNorm(h)))). Spatial: `frames` frames [frames*H*W, C], at most the frame
 * chunk (LC_ERR_NOMEM beyond), queries in token chunks; the V third of q,k,v goes from the projection's
 * epilogue straight into the transposed layout the attention kernel stages. Temporal: all B*F frames
 * [B*F*H*W, C], in position chunks. */
lc_status lc_op_spatial_block(lc_ctx* ctx, void* h, int frames);
lc_status lc_op_temporal_block(lc_ctx* ctx, void* h);
/* Spatial attention core: per frame and head, softmax(QK^T/sqrt(d))V over the H*W tokens of the
 * frame, for query tokens [q0, q1). qkv [frames*H*W, 3C] -> out [frames*H*W, C]; rows of other
 * queries are not written. q_prescaled: 0 = the q third holds Q; 1 = it holds Q*log2(e)/sqrt(d). */
lc_status lc_op_spatial_attention(lc_ctx* ctx, const void* qkv, void* out, int frames, int q0, int q1,
                                  int q_prescaled);
/* Temporal attention core: qkv [(B*F) * positions, 3C] (frame-major) -> out [(B*F)*positions, C];
 * per batch element, position and head attention over the F frames. */
lc_status lc_op_temporal_attention(lc_ctx* ctx, const void* qkv, void* out, int positions);
/* y[rows, C] (float) = res (float) + a[rows, C] Wo^T + bo of LC_L_SATTN / LC_L_TATTN. res may be
 * NULL or equal y. */
lc_status lc_op_proj(lc_ctx* ctx, int layer, const void* a, const void* res, void* y, int64_t rows);
/* d0[frames*(H/2)*(W/2), C_deep] (float) = stride-2 conv3x3 of x[frames*H*W, C] (float): the first
 * half of the deep stand-in of the normal step. */
lc_status lc_op_down_conv(lc_ctx* ctx, const void* x, void* d0, int frames);
/* u[frames*H*W, C] (float) = conv3x3(SiLU(GroupNorm(Concat(skip, up2(deep))))) ([FC]); skip float
 * [frames*H*W, C], deep cfg dtype [frames*(H/2)*(W/2), C_deep] (a cache entry, channels-last). */
lc_status lc_op_up_conv(lc_ctx* ctx, const void* skip, const void* deep, void* u, int frames);
/* eps[frames, C_lat, H, W] (cfg dtype) = conv_out(SiLU(GroupNorm(u))), u float [frames*H*W, C]. */
lc_status lc_op_conv_out(lc_ctx* ctx, const void* u, void* eps, int frames);

/* ---- sliced decoding ("Feature chunk and Sliced Decoding" section) --------------------------------------------
 * At the decoding stage the batch and frame axes are merged (F in R^{(B x T) x C x H x W}) and the decoder would
 * take all frames at once; sliced decoding decodes the latent video `slice_frames` frames at a time (1 = frame by
 * frame) and merges the images back in frame order. Every operator of the decoder works on one frame at a time, so
 * the result does not depend on the slice size (bit for bit), and the workspace is sized by the slice.
 * The paper uses its models' pretrained decoders and does not describe them; this is a stand-in of the usual shape:
 *   conv_in 3x3 C_lat -> widths[0]; ResBlock, spatial self-attention block, ResBlock at widths[0];
 *   level l = 0 .. levels-1: ResBlock(widths[l]), nearest 2x upsampling, conv3x3 widths[l] -> widths[l+1];
 *   GroupNorm -> SiLU -> conv3x3 widths[levels] -> C_img.
 * ResBlock(h) = h + conv3x3(SiLU(GroupNorm(h))); the attention block is h + proj(Attn(qkv(GroupNorm(h)))) with
 * bias-free q/k/v, `heads` heads of `head_dim`, scale 1/sqrt(head_dim), output projection with bias. It runs on
 * the kernels of the denoising stage. Calls only enqueue on the stream given at creation; lc_decoder_sync drains it.
 * Requirements (else LC_ERR_SHAPE): sizes > 0; 0 <= levels <= LC_DEC_MAX_LEVELS; widths multiples of 64, <= 1024,
 * divisible by groups; heads * head_dim == widths[0]; head_dim in {8, 16, 32, 40, 64}; C_lat <= 16; C_img <= 32. */
#define LC_DEC_MAX_LEVELS 3
typedef struct lc_decoder lc_decoder; /* opaque; owned by the library */
typedef struct lc_decoder_config {
  int32_t N, H, W;       /* frames (batch x frames merged), latent size */
  int32_t C_lat, C_img;  /* latent channels, image channels */
  int32_t levels;        /* 2x upsampling levels: images are H * 2^levels x W * 2^levels */
  int32_t widths[LC_DEC_MAX_LEVELS + 1];
  int32_t groups, heads, head_dim;
  int32_t dtype;         /* lc_dtype of z, the images and the weights */
  float gn_eps;
} lc_decoder_config;
/* all [device], cfg dtype, PyTorch layouts; packed private copies are made by lc_decoder_load_weights */
typedef struct lc_decoder_weights {
  const void *conv_in_w, *conv_in_b;
  lc_gnconv_w mid_res[2];
  lc_attn_w mid_attn;
  lc_gnconv_w up_res[LC_DEC_MAX_LEVELS];
  const void *up_conv_w[LC_DEC_MAX_LEVELS], *up_conv_b[LC_DEC_MAX_LEVELS];
  lc_gnconv_w out; /* GroupNorm(widths[levels]) -> SiLU -> conv widths[levels] -> C_img */
} lc_decoder_weights;

lc_status lc_decoder_check_config(const lc_decoder_config* cfg);                     /* host only */
/* Workspace a pass over slice_frames frames needs (0 or > N: all N frames): two maps of the largest stage per
 * frame of the slice, statistics, and the attention block's q,k,v. 0 if cfg is invalid. Host only. */
size_t lc_decoder_workspace_bytes(const lc_decoder_config* cfg, int slice_frames);
const char* lc_decoder_last_error(const lc_decoder* dec);
/* stream: hipStream_t owned by the caller, must outlive the decoder. */
lc_status lc_decoder_create(const lc_decoder_config* cfg, void* stream, lc_decoder** out);
lc_status lc_decoder_destroy(lc_decoder* dec);
lc_status lc_decoder_load_weights(lc_decoder* dec, const lc_decoder_weights* w /* [host] struct of [device] ptrs */);
/* arena: [device], 256-byte aligned, caller-owned; must cover lc_decoder_workspace_bytes of the slices used. */
lc_status lc_decoder_set_workspace(lc_decoder* dec, void* arena, size_t bytes);
/* z [device, N, C_lat, H, W] -> img [device, N, C_img, H * 2^levels, W * 2^levels], in passes of slice_frames
 * frames. LC_ERR_NOMEM if the workspace is too small for that slice; LC_ERR_STATE without weights / workspace.
 * z and img must stay valid until the stream has been synchronised. */
lc_status lc_decode(lc_decoder* dec, const void* z, void* img, int slice_frames);
lc_status lc_decoder_sync(lc_decoder* dec);

/* ---- diffusion-transformer variant --------------------------------------------------------------------------
 * The reuse rule of [AS] applied to a stack of L adaLN-modulated transformer blocks over the B x T tokens of a
 * video (T = all patches of all latent frames: full 3-D attention per batch element). Blocks [cache_a, cache_b)
 * are the cached deep part: what they add to the hidden states, Delta = x_b - x_a, is accumulated in a device slot
 * at a normal step (lc_dit_full_step), swapped to pinned host memory and back like the U-Net's deep feature, and
 * added back at a cache step (lc_dit_cached_step), which runs only blocks [0, cache_a) and [cache_b, L). In both
 * kinds of step the deep part enters as x_a + Delta, so a cache step on the Delta of the same input reproduces the
 * normal step bit for bit. The paper does not say which blocks of a DiT are cached; this split is a reading.
 * One block: h = LN(x) (1 + scale_msa) + shift_msa; x += gate_msa * (Attn(h) Wo^T + bo); h = LN(x) (1 + scale_mlp)
 * + shift_mlp; x += gate_mlp * (W2 gelu_tanh(W1 h + b1) + b2). LN: per token, biased variance, no affine; q,k,v
 * projections with bias; `heads` heads of `head_dim`, scale 1/sqrt(head_dim). The modulation vectors are inputs.
 * Feature chunk ([CHK]): token_chunk of the B*T tokens of a step per pass of LayerNorm / projections / MLP (a pass may
 * run across batch elements: every row looks up its own modulation) and min(token_chunk, T) queries of every batch
 * element per pass of the attention (against all keys); it never changes results. Hidden states and modulation are float at the boundary;
 * weights have cfg dtype (bf16: MFMA operands bf16, accumulation and the residual stream fp32).
 * Requirements (else LC_ERR_SHAPE): sizes > 0; D a multiple of 64, <= 2048; heads * head_dim == D; head_dim in
 * {8, 16, 32, 40, 64}; L <= LC_DIT_MAX_BLOCKS; 0 <= cache_a <= cache_b <= L; mlp_ratio <= 8; 1 <= dev_slots <= 8;
 * 0 <= host_slots <= 64. Conventions (streams, errors, lifetimes) as for the U-Net stage. */
#define LC_DIT_MAX_BLOCKS 64
typedef struct lc_dit lc_dit; /* opaque; owned by the library */
typedef struct lc_dit_config {
  int32_t B, T, D, heads, head_dim;
  int32_t L, cache_a, cache_b, mlp_ratio;
  int32_t dtype;  /* lc_dtype of the weights and of the MFMA operands */
  float ln_eps;
  int32_t host_slots, dev_slots;
} lc_dit_config;
/* [device], cfg dtype, PyTorch layouts: wqkv [3D, D] (q, k, v rows stacked), wo [D, D], w1 [mlp_ratio*D, D],
 * w2 [D, mlp_ratio*D], biases [out]. Private copies are made by lc_dit_load_weights. */
typedef struct lc_dit_block_w { const void *wqkv, *bqkv, *wo, *bo, *w1, *b1, *w2, *b2; } lc_dit_block_w;
typedef struct lc_dit_weights { lc_dit_block_w blk[LC_DIT_MAX_BLOCKS]; } lc_dit_weights;

lc_status lc_dit_check_config(const lc_dit_config* cfg);                 /* host only */
size_t lc_dit_entry_bytes(const lc_dit_config* cfg);                     /* one Delta entry: B*T*D floats; host only */
size_t lc_dit_workspace_bytes(const lc_dit_config* cfg, int token_chunk); /* footprint model; host only */
const char* lc_dit_last_error(const lc_dit* ctx);
lc_status lc_dit_create(const lc_dit_config* cfg, void* compute_stream, void* side_stream, lc_dit** out);
lc_status lc_dit_destroy(lc_dit* ctx);
lc_status lc_dit_load_weights(lc_dit* ctx, const lc_dit_weights* w /* [host] struct of [device] ptrs */);
lc_status lc_dit_set_workspace(lc_dit* ctx, void* arena /* [device], 256-byte aligned */, size_t bytes);
lc_status lc_dit_set_chunk(lc_dit* ctx, int token_chunk); /* 0 = unchunked; values above B*T clamp */
/* x_in, x_out [device, B, T, D] float; mod [device, L, B, 6, D] float in the order shift_msa, scale_msa, gate_msa,
 * shift_mlp, scale_mlp, gate_mlp. Normal step: all L blocks, Delta left in device slot dev_slot. Cache step: Delta
 * read from dev_slot (LC_ERR_STATE if empty; waits on the GPU for a swap-in in flight). */
lc_status lc_dit_full_step(lc_dit* ctx, const void* x_in, const void* mod, void* x_out, int dev_slot);
lc_status lc_dit_cached_step(lc_dit* ctx, const void* x_in, const void* mod, void* x_out, int dev_slot);
lc_status lc_dit_swap_out(lc_dit* ctx, int dev_slot, int host_slot); /* async D2H on the side stream */
lc_status lc_dit_swap_in(lc_dit* ctx, int host_slot, int dev_slot);  /* async H2D on the side stream */
lc_status lc_dit_sync(lc_dit* ctx);
lc_status lc_dit_cache_write(lc_dit* ctx, int dev_slot, const void* delta /* [device, B, T, D] float */);
lc_status lc_dit_cache_peek(lc_dit* ctx, int host_slot, const void** ptr /* [host] */, size_t* bytes);
lc_status lc_dit_cache_dev_peek(lc_dit* ctx, int dev_slot, const void** ptr /* [device] */, size_t* bytes);
lc_status lc_dit_get_counts(lc_dit* ctx, int64_t* full_steps, int64_t* cached_steps, int64_t* swaps_out, int64_t* swaps_in);

/* ---- U-Net stage with real block internals -------------------------------------------------------------------
 * The normal and the cache step of [FC] / [AS] on a U-Net whose blocks are those of the video U-Nets the paper ran
 * (it takes them from its pretrained models and does not describe them; synthetic weights here) and whose deep
 * branch has three levels, so that the refresh interval of [AS] can be swept end to end:
 *   RB(x; temb)  h = conv1(SiLU(GN(x))) + (W_t SiLU(temb) + b_t)[channel];  y = short(x) + conv2(SiLU(GN(h)));
 *                short = identity, or a 1x1 convolution when the channel count changes
 *   ST(x; ctx)   z = pin(GN(x)); z += SelfAttn(LN(z)); z += CrossAttn(LN(z), ctx); z += FF(LN(z)); y = x + pout(z);
 *                tokens = the positions of one frame; FF(h) = W2 (a * gelu_tanh(g)) + b2 with [a, g] = W1 h + b1
 *   TT(x)        z = pin(GN(x)); z += SelfAttn(LN(z) + PE); z += FF(LN(z)); y = x + pout(z); tokens = the F frames of
 *                one position; PE[f, 2i] = sin(f / 10000^(2i/C)), PE[f, 2i+1] = cos(f / 10000^(2i/C))
 *   shallow down s = TT(ST(RB(conv_in(x))))                                  C  at H x W
 *   deep         d = TT(ST(RB(Down(s))));  e = UpC(RB(RB(Down(d))));         C1 at H/2 x W/2, C2 at H/4 x W/4
 *                d = TT(ST(RB(Concat(d, e))));  deep = UpC(d)                the cached feature: C1 at H x W
 *   shallow up   u = TT(ST(RB(Concat(s, deep))));  eps = conv_out(SiLU(GN(u)))
 * Down = conv3x3 stride 2, UpC = conv3x3 after nearest 2x upsampling; attention: bias-free q/k/v, heads of head_dim
 * channels (C / head_dim and C1 / head_dim heads), scale 1/sqrt(head_dim), output projection with bias; LayerNorm with
 * affine. A normal step (lc_unet_full_step) runs everything and leaves `deep` in a device slot; a cache step
 * (lc_unet_cached_step) runs the shallow blocks only and reads it from the slot. Entries are fp32, channels-last
 * [B*F, H*W, C1]; swap-out / swap-in move them to / from pinned host memory on the side stream, as for the stage
 * above. x, temb, ctx, eps and the weights have cfg dtype (bf16: MFMA operands bf16, accumulation and residual
 * streams fp32).
 * Feature chunk ("Feature chunk" section): lc_unet_set_chunk(frame_chunk) makes every block work on a chunk at a
 * time. The residual blocks, the spatial transformer blocks and the resampling convolutions, which treat frames
 * independently, take frame_chunk of the B*F frames at H x W and twice as many at each level down (a frame there has
 * a quarter of the positions and twice the channels: a chunk's maps keep their size); a temporal block, whose tokens
 * are the frames of a position, takes ceil(positions * chunk frames / (B*F)) positions of every frame (the same number
 * of rows) and never splits the frame axis. What lives inside a block (the concatenated input, hidden map and shortcut of a residual block,
 * the upsampled map, the token buffers of a transformer block) then has the size of one chunk; what passes
 * between blocks (three maps, the two skips, the device slots) keeps the size of all frames. Results are the same
 * bit for bit at every setting.
 * Requirements (else LC_ERR_SHAPE): sizes > 0; H, W multiples of 4; C, C1, C2, ctx_dim multiples of 64, <= 2048;
 * every width and C + C1, C1 + C2 divisible by groups; C, C1 multiples of head_dim; head_dim in {8, 16, 32, 40, 64};
 * C_lat <= 16; ff_mult <= 4; F * 3 * max(C, C1) elements of cfg dtype within 128 KiB (one position's q,k,v of all
 * frames in LDS); 1 <= dev_slots <= 8; 0 <= host_slots <= 64. Conventions (streams, errors, lifetimes) as above. */
typedef struct lc_unet lc_unet; /* opaque; owned by the library */
typedef struct lc_unet_config {
  int32_t B, F, H, W, C_lat;
  int32_t C, C1, C2;       /* widths at H x W, H/2 x W/2, H/4 x W/4 */
  int32_t groups, head_dim;
  int32_t ctx_len, ctx_dim; /* conditioning tokens per batch element and their width */
  int32_t temb_dim, ff_mult;
  int32_t dtype;
  float gn_eps, ln_eps;
  int32_t host_slots, dev_slots;
} lc_unet_config;
/* all [device], cfg dtype, PyTorch layouts ([out, in] / [out, in, 3, 3]); short_w / short_b NULL when Cin == Cout */
typedef struct lc_unet_rb_w {
  const void *gn1_g, *gn1_b, *conv1_w, *conv1_b, *temb_w, *temb_b, *gn2_g, *gn2_b, *conv2_w, *conv2_b, *short_w, *short_b;
} lc_unet_rb_w;
typedef struct lc_unet_attn_w { const void *wq, *wk, *wv, *wo, *bo; } lc_unet_attn_w;
/* attn2 (cross-attention: wk, wv are [C, ctx_dim]) and ln2 are NULL in a temporal block */
typedef struct lc_unet_tf_w {
  const void *gn_g, *gn_b, *pin_w, *pin_b, *ln1_g, *ln1_b;
  lc_unet_attn_w attn1;
  const void *ln2_g, *ln2_b;
  lc_unet_attn_w attn2;
  const void *ln3_g, *ln3_b, *ff1_w, *ff1_b, *ff2_w, *ff2_b, *pout_w, *pout_b;
} lc_unet_tf_w;
typedef struct lc_unet_conv_w { const void *w, *b; } lc_unet_conv_w;
typedef struct lc_unet_weights {
  lc_unet_conv_w conv_in;
  lc_unet_rb_w rb[6];   /* d0 (C -> C), d1 (C -> C1), mid0 (C1 -> C2), mid1 (C2 -> C2), u1 (C1 + C2 -> C1), u0 (C + C1 -> C) */
  lc_unet_tf_w st[4];   /* d0 (C), d1 (C1), u1 (C1), u0 (C) */
  lc_unet_tf_w tt[4];   /* the same places */
  lc_unet_conv_w down[2]; /* d0 (C), d1 (C1) */
  lc_unet_conv_w up[2];   /* u2 (C2), u1 (C1) */
  const void *out_gn_g, *out_gn_b;
  lc_unet_conv_w out;   /* C -> C_lat */
} lc_unet_weights;

lc_status lc_unet_check_config(const lc_unet_config* cfg);   /* host only */
size_t lc_unet_entry_bytes(const lc_unet_config* cfg);       /* one cache entry: B*F*H*W*C1 floats; host only */
size_t lc_unet_workspace_bytes(const lc_unet_config* cfg);   /* footprint model, device slots included, all frames at
                                                                 once (the largest over all chunk settings); host only */
size_t lc_unet_chunk_workspace_bytes(const lc_unet_config* cfg, int frame_chunk); /* the same at a chunk setting */
const char* lc_unet_last_error(const lc_unet* ctx);
lc_status lc_unet_create(const lc_unet_config* cfg, void* compute_stream, void* side_stream, lc_unet** out);
lc_status lc_unet_destroy(lc_unet* ctx);
lc_status lc_unet_load_weights(lc_unet* ctx, const lc_unet_weights* w /* [host] struct of [device] ptrs */);
lc_status lc_unet_set_workspace(lc_unet* ctx, void* arena /* [device], 256-byte aligned */, size_t bytes);
/* 0 = all frames at once; values above B*F clamp. LC_ERR_NOMEM if the workspace at hand is smaller than the setting
 * needs. The device slots keep their place and contents. Not while a step is in flight. */
lc_status lc_unet_set_chunk(lc_unet* ctx, int frame_chunk);
/* x [device, B, F, C_lat, H, W], temb [device, B, temb_dim], ctx [device, B, ctx_len, ctx_dim] -> eps [device, B, F,
 * C_lat, H, W], all of cfg dtype. Cache step: LC_ERR_STATE if the slot is empty; waits on the GPU for a swap-in in
 * flight. All four tensors must stay valid until the compute stream has been synchronised. */
lc_status lc_unet_full_step(lc_unet* ctx, const void* x, const void* temb, const void* cond, void* eps, int dev_slot);
lc_status lc_unet_cached_step(lc_unet* ctx, const void* x, const void* temb, const void* cond, void* eps, int dev_slot);
lc_status lc_unet_swap_out(lc_unet* ctx, int dev_slot, int host_slot); /* async D2H on the side stream */
lc_status lc_unet_swap_in(lc_unet* ctx, int host_slot, int dev_slot);  /* async H2D on the side stream */
lc_status lc_unet_sync(lc_unet* ctx);
lc_status lc_unet_cache_write(lc_unet* ctx, int dev_slot, const void* deep /* [device, B*F, H*W, C1] float */);
lc_status lc_unet_cache_peek(lc_unet* ctx, int host_slot, const void** ptr /* [host] */, size_t* bytes);
lc_status lc_unet_cache_dev_peek(lc_unet* ctx, int dev_slot, const void** ptr /* [device] */, size_t* bytes);

#ifdef __cplusplus
}
#endif
#endif /* LIGHTCACHE_H */
