/*
 * cfdetr.h - C ABI of the MI355X coarse-to-fine detection-transformer encoder.
 *
 * The library computes the data-parallel part of CF-DETR (Sec. III-B of the
 * paper, strategies A1-A3):
 *   A1  coarse inference: every camera frame is cut into a coarse grid of
 *       patches, each patch becomes one token, and the transformer encoder
 *       (self-attention among all tokens of a frame, Sec. II-A) runs on an
 *       image-level batch of frames;
 *   A2  selective fine inference: only the regions of interest are
 *       re-partitioned into finer patches; everywhere else the coarse-stage
 *       tokens are reused, which yields a mixed-granularity token set;
 *   A3  multi-level batch inference: the token sets of several frames, of
 *       different lengths, go through the encoder together.  The paper pads
 *       them to one length; this library keeps them as variable-length
 *       sequences addressed by offsets, which computes the same thing without
 *       the padding work.
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer (gfx950) owned by the caller,
 *     unless a parameter says "host".  Frames, boxes, weights and the fp32
 *     token/output buffers must be 16-byte aligned (else CFDETR_EINVAL).  The library never frees or keeps
 *     ownership of caller memory.  Weights must outlive the context and must
 *     not change while it exists: some kernels read private re-ordered copies
 *     of the matrices that cfdetr_create makes.
 *   - Work space is allocated once in cfdetr_create from the max_* fields and
 *     released in cfdetr_destroy; the encode calls allocate nothing.
 *   - Calls enqueue work on the given hipStream_t (passed as void*; NULL is
 *     the default stream) and return without waiting.  No call synchronises
 *     the host except cfdetr_sync_status, cfdetr_profile_end and
 *     cfdetr_create / cfdetr_destroy.
 *   - One context serves one stream at a time; calls on one context must not
 *     overlap.  Different contexts are independent.
 *   - Host-detectable argument errors return a status at once and enqueue
 *     nothing.  A token total that exceeds max_tokens_total is detected on the
 *     device: the selection then reports zero tokens for every frame, raises a
 *     sticky flag, and cfdetr_sync_status returns CFDETR_ECAPACITY.  Output is
 *     never silently truncated.
 *
 * Token descriptor: one int32 per token, level<<28 | row<<14 | col, where
 * (row, col) index the grid of that level (level 0 = coarsest).
 * Token order: frames in batch order; inside a frame coarse level first, and
 * row-major inside a level.
 *
 * Number formats: matrices are stored in act_dtype (bf16 bit patterns or
 * fp32); bias and LayerNorm vectors are always fp32; frames are stored in
 * image_dtype; the cached coarse tokens (x0_cache) and both encoder outputs are
 * always fp32.  With act_dtype = CFDETR_BF16 all contractions run on bf16
 * matrix cores with fp32 accumulation and fp32 softmax / LayerNorm / residual
 * stream; CFDETR_FP32 is a slow all-fp32 check mode.
 */
#ifndef CFDETR_H
#define CFDETR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CFDETR_API __attribute__((visibility("default")))

typedef struct cfdetr_ctx cfdetr_ctx; /* opaque; owns work space only */

typedef enum {
  CFDETR_OK = 0,
  CFDETR_EINVAL = 1,    /* null pointer, bad enum, bad field value             */
  CFDETR_ESHAPE = 2,    /* shape constraint violated (see cfdetr_config)       */
  CFDETR_ECAPACITY = 3, /* batch / token / box count beyond the configured max */
  CFDETR_ENOMEM = 4,    /* device or host allocation failed                    */
  CFDETR_EDEVICE = 5    /* a HIP call failed; see cfdetr_last_error            */
} cfdetr_status;

typedef enum { CFDETR_BF16 = 0, CFDETR_FP32 = 1 } cfdetr_dtype;

#define CFDETR_MAX_LEVELS 3

/*
 * Shape of the model and capacity of the work space.
 * Constraints (else CFDETR_ESHAPE): n_levels in {1,2,3}; patch[l] = patch[l-1]/2;
 * patch[n_levels-1] >= 8; img_h, img_w multiples of patch[0]; every grid at
 * most 16384 cells per side; d_model a multiple of 64 and of n_heads;
 * d_model / n_heads in {32, 64}; d_ffn a multiple of 64; n_layers >= 1;
 * 1 <= max_batch <= 64; max_tokens_total >= max_batch * (coarse cells).
 */
typedef struct {
  int32_t n_levels;
  int32_t patch[CFDETR_MAX_LEVELS]; /* coarse -> fine, in pixels */
  int32_t img_h, img_w;
  int32_t d_model, n_heads, n_layers, d_ffn;
  int32_t max_batch;        /* frames per call                                  */
  int32_t max_tokens_total; /* tokens per call over all frames (fine pass)      */
  cfdetr_dtype image_dtype; /* element type of the frames                       */
  cfdetr_dtype act_dtype;   /* element type of weight matrices and contractions */
  float ln_eps;             /* LayerNorm epsilon, e.g. 1e-5                     */
} cfdetr_config;

/*
 * Encoder weights (device pointers).  Layouts, all row-major:
 *   w_embed[l] [d_model, 3*patch[l]^2]  patch flattened (channel, row, column)
 *   b_embed[l] [d_model]
 *   per layer, stacked over layers in the leading dimension:
 *   ln1_g, ln1_b [L, d]      w_qkv [L, 3d, d] (query rows, key rows, value rows;
 *   b_qkv [L, 3d]            head h owns rows h*dh..(h+1)*dh of each third)
 *   w_o [L, d, d]  b_o [L, d]  ln2_g, ln2_b [L, d]
 *   w_ff1 [L, d_ffn, d]  b_ff1 [L, d_ffn]  w_ff2 [L, d, d_ffn]  b_ff2 [L, d]
 *   lnf_g, lnf_b [d]         final LayerNorm
 * Each layer is pre-LN: x += Wo.MHA(LN1 x); x += W2.GELU(W1.LN2 x); the output
 * is LNf(x) after the last layer.
 */
typedef struct {
  const void* w_embed[CFDETR_MAX_LEVELS];
  const float* b_embed[CFDETR_MAX_LEVELS];
  const float *ln1_g, *ln1_b;
  const void* w_qkv;
  const float* b_qkv;
  const void* w_o;
  const float* b_o;
  const float *ln2_g, *ln2_b;
  const void* w_ff1;
  const float* b_ff1;
  const void* w_ff2;
  const float* b_ff2;
  const float *lnf_g, *lnf_b;
} cfdetr_weights;

/* Kernel families, for cfdetr_profile_end. */
typedef enum {
  CFDETR_K_SELECT = 0, /* A2 cell tests, compaction, offsets                   */
  CFDETR_K_PLAN = 1,   /* attention work list from the sequence offsets        */
  CFDETR_K_EMBED = 2,  /* patch gather + projection + position                 */
  CFDETR_K_GATHER = 3, /* reuse of cached coarse tokens                        */
  CFDETR_K_LN = 4,     /* LayerNorm                                            */
  CFDETR_K_QKV = 5,    /* query/key/value projection                           */
  CFDETR_K_ATTN = 6,   /* variable-length self-attention                       */
  CFDETR_K_OUT = 7,    /* output projection + residual                         */
  CFDETR_K_FF1 = 8,    /* first FFN projection + GELU                          */
  CFDETR_K_FF2 = 9,    /* second FFN projection + residual; where one kernel does
                          everything of a layer after attention, that kernel      */
  CFDETR_K_ROI = 10,   /* difficulty test and region proposal                  */
  CFDETR_K_DEC = 11,   /* decoder kernels that are not one of the families above
                          (cast, query broadcast, key/value projection, heads)   */
  CFDETR_K_COUNT = 12
} cfdetr_kernel_id;

/* Host-side.  Validates cfg, copies it, keeps the weight POINTERS, allocates
 * the work space on the current device and builds the position tables there.
 * For d_model 256 in bf16 with d_ffn a multiple of 128 up to 2048 it also
 * copies w_qkv, w_o, w_ff1, w_ff2 into the order its fused layer kernels read
 * (the weights are read once, here).
 * On failure *out is NULL. */
CFDETR_API cfdetr_status cfdetr_create(const cfdetr_config* cfg, const cfdetr_weights* w,
                            cfdetr_ctx** out);
/* Waits for the device, frees the work space.  NULL is allowed. */
CFDETR_API void cfdetr_destroy(cfdetr_ctx* ctx);
/* Host string describing the last error on this context ("" if none).  With
 * ctx == NULL: the reason the calling thread's last cfdetr_create failed.  The
 * pointer stays valid until the next failing call. */
CFDETR_API const char* cfdetr_last_error(const cfdetr_ctx* ctx);
/* Bytes of device work space the context holds. */
CFDETR_API uint64_t cfdetr_workspace_bytes(const cfdetr_ctx* ctx);
/* Waits for `hip_stream`, then reports and clears the device-side sticky flag:
 * CFDETR_OK, or CFDETR_ECAPACITY if a selection overflowed max_tokens_total. */
CFDETR_API cfdetr_status cfdetr_sync_status(cfdetr_ctx* ctx, void* hip_stream);

/*
 * A1, coarse inference on an image-level batch (Sec. III-B, A1).
 *   images   [B, 3, img_h, img_w] in image_dtype, planar
 *   x0_cache [B*N0, d] fp32 out: the coarse tokens as they enter the encoder
 *            (patch projection + position); may be NULL if not wanted
 *   y_coarse [B*N0, d] fp32 out: encoder output, frame after frame, row-major grid
 * N0 = (img_h/patch[0]) * (img_w/patch[0]).  1 <= B <= max_batch.
 */
CFDETR_API cfdetr_status cfdetr_coarse_encode(cfdetr_ctx* ctx, const void* images, int32_t B,
                                   float* x0_cache, float* y_coarse, void* hip_stream);

/*
 * Parameters of the difficulty test and the region proposal (host memory).
 * Sec. III-B quotes tau_hi = 0.8 and tau_lo = 0.05 as examples.
 */
typedef struct {
  float tau_hi;   /* a query with confidence above this is a certain, prominent object */
  float tau_lo;   /* a frame is easy iff the average confidence of its other queries is
                     below this; queries in (tau_lo, tau_hi] propose regions          */
  float scale;    /* a region is the query's box scaled by this about its centre (1 = box) */
  float min_side; /* least width and height of a region, in pixels (0 = none)          */
  int32_t tier;   /* refinement level the regions ask for, 0..n_levels-1               */
} cfdetr_roi_params;

/*
 * A1 difficulty test and A2 region proposal from the coarse stage's object queries
 * (Sec. III-B, A1: queries above tau_hi are left out, the confidences of the others
 * are averaged, a frame whose average is below tau_lo is easy and skips the fine
 * stage; A2: the regions of a hard frame come from the location and size of its
 * queries of intermediate confidence).
 *   queries     [B, Q, 5] fp32 (cx, cy, w, h, c): centre and size of the candidate
 *               box as fractions of the frame, confidence in [0, 1]; finite values;
 *               16-byte aligned; 1 <= Q <= 65536
 *   params      host pointer; tau_lo <= tau_hi, scale >= 0, min_side >= 0
 *   max_boxes   capacity of boxes / tier
 * Outputs (device), in the form cfdetr_select_fine takes:
 *   boxes       [max_boxes, 4] int32 half-open pixel rectangles, smallest cover of the
 *               scaled box, clipped to the frame; frame after frame, query order
 *   tier        [max_boxes] uint8, params->tier for every region
 *   box_offsets [B+1] int32
 *   hard        [B] int32: 1 = hard; an easy frame proposes no region
 *   mean_conf   [B] fp32: the average that decided it (0 if no query was left)
 * Decisions are taken in fp64 on the fp32 inputs.  More than max_boxes regions in
 * total: nothing is proposed (all offsets 0), a sticky flag is raised and
 * cfdetr_sync_status returns CFDETR_ECAPACITY.
 */
CFDETR_API cfdetr_status cfdetr_propose_rois(cfdetr_ctx* ctx, const float* queries, int32_t B,
                                  int32_t Q, const cfdetr_roi_params* params,
                                  int32_t max_boxes, int32_t* boxes, uint8_t* tier,
                                  int32_t* box_offsets, int32_t* hard, float* mean_conf,
                                  void* hip_stream);

/*
 * End of A2 (Sec. III-B): the final detections of every frame.  Confident coarse
 * detections are kept, and in a hard frame the fine stage's detections take the place of
 * the uncertain ones.  The paper fixes no more than that; this library's reading: frame f
 * keeps its coarse-stage queries with c > tau_hi, in query order, and, if hard[f] != 0,
 * then adds its fine-stage queries with c > tau_fine, in query order.  An easy frame has
 * no fine stage: its rows of `fine` are not read for a decision.
 *   coarse, fine [B, Q, 5] fp32 (cx, cy, w, h, c), e.g. from cfdetr_decode of y_coarse / y_mixed
 *   hard   [B] int32, as cfdetr_propose_rois writes it
 *   det    [B, 2Q, 5] fp32 out: the detections of frame f in rows 0 .. count[f]; the other
 *          rows are cleared to 0
 *   src    [B, 2Q] uint8 out: 0 = from the coarse stage, 1 = from the fine stage, 255 past
 *          the count
 *   count  [B] int32 out
 * Values are copied unchanged.  1 <= Q <= 65536; tau_hi and tau_fine must not be NaN.
 */
CFDETR_API cfdetr_status cfdetr_merge_detections(cfdetr_ctx* ctx, const float* coarse,
                                     const float* fine, const int32_t* hard, int32_t B,
                                     int32_t Q, float tau_hi, float tau_fine, float* det,
                                     uint8_t* src, int32_t* count, void* hip_stream);

/*
 * A2, selective patch split as integer work only (Sec. III-B, A2).
 *   boxes       [n_boxes, 4] int32 (x0, y0, x1, y1), half-open pixel rectangles;
 *               clipped to the frame; empty ones select nothing
 *   tier        [n_boxes] uint8: finest level this box asks for (0 = not
 *               critical, n_levels-1 = finest); larger values act as finest
 *   box_offsets [B+1] int32: boxes of frame i are box_offsets[i]..box_offsets[i+1]
 * A cell of a non-finest level l is replaced by its four children iff a box of
 * the same frame with tier > l overlaps it; the unsplit cells are the tokens.
 * Outputs:
 *   tok_desc     [max_tokens_total] int32; entries past the total are untouched
 *   cu_seqlens   [B+1] int32: token offsets of the frames, cu_seqlens[0] = 0
 *   level_counts [B, n_levels] int32: tokens of frame i at each level; may be NULL
 */
CFDETR_API cfdetr_status cfdetr_select_fine(cfdetr_ctx* ctx, const int32_t* boxes, const uint8_t* tier,
                                 const int32_t* box_offsets, int32_t B, int32_t* tok_desc,
                                 int32_t* cu_seqlens, int32_t* level_counts,
                                 void* hip_stream);

/*
 * cfdetr_select_fine with the outcome of the difficulty test (Sec. III-B, A1: an easy
 * frame is done after the coarse stage and its fine-grained processing is skipped).
 *   hard  [B] int32 (device), as cfdetr_propose_rois writes it: a frame with hard[f] == 0
 *         gets no token at all: cu_seqlens[f+1] == cu_seqlens[f], its level_counts are 0,
 *         and cfdetr_fine_encode computes and writes nothing for it.
 * Everything else as in cfdetr_select_fine (which keeps such a frame in the batch as a
 * coarse-only token set, whose result equals its coarse result).
 */
CFDETR_API cfdetr_status cfdetr_select_fine_hard(cfdetr_ctx* ctx, const int32_t* boxes,
                                      const uint8_t* tier, const int32_t* box_offsets,
                                      const int32_t* hard, int32_t B, int32_t* tok_desc,
                                      int32_t* cu_seqlens, int32_t* level_counts,
                                      void* hip_stream);

/*
 * cfdetr_select_fine for callers that cannot allocate device memory and have no context:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * call allocates nothing and needs no cfdetr_create: its scratch memory (one flag byte per
 * frame and cell of the levels below the finest) is a static device array of 1 MiB that
 * every GPU the library runs on holds until the process ends.
 *   cfg       host pointer; the same structure cfdetr_create takes (its pyramid fields,
 *             max_batch and max_tokens_total are used; all fields are validated)
 *   overflow  [1] int32 (device) out: 0, or 1 if the token total exceeds
 *             cfg->max_tokens_total; then cu_seqlens and level_counts are all 0 and
 *             tok_desc is untouched (there is no context to hold a sticky flag)
 *   other arguments and outputs exactly as in cfdetr_select_fine, bit for bit.
 * Limits: B * (cells of all levels but the finest) <= 1048576, else CFDETR_ECAPACITY and
 * nothing is enqueued.  The reason for a failure is cfdetr_last_error(NULL).
 * All calls on one GPU share the one array, which keeps the last call's contents (each call
 * clears what it uses, with a kernel): calls that overlap on one GPU, on whatever streams or
 * threads, race.  Calls in stream order on one stream are safe.
 */
CFDETR_API cfdetr_status cfdetr_select_fine_static(const cfdetr_config* cfg, const int32_t* boxes,
                                        const uint8_t* tier, const int32_t* box_offsets,
                                        int32_t B, int32_t* tok_desc, int32_t* cu_seqlens,
                                        int32_t* level_counts, int32_t* overflow,
                                        void* hip_stream);

/*
 * A2 + A3, encoder over the mixed-granularity token sets as one variable-length
 * batch (Sec. III-B, A2 "reuse the coarse-stage tokens", A3 patch-level batch).
 *   images, B    as in cfdetr_coarse_encode
 *   tok_desc, cu_seqlens  as written by cfdetr_select_fine (device)
 *   x0_cache     [B*N0, d] fp32 from cfdetr_coarse_encode on the same frames:
 *                level-0 tokens are copied from it; NULL embeds them again
 *   y_mixed      [max_tokens_total, d] fp32 out; rows past cu_seqlens[B] untouched
 * Attention stays inside [cu_seqlens[i], cu_seqlens[i+1]) for every frame i.  A frame may
 * have no token (cu_seqlens[i+1] == cu_seqlens[i]): nothing is computed for it.
 * The offsets are checked on the device before anything reads them: a negative length
 * or a total above max_tokens_total makes the call compute and write nothing, and
 * cfdetr_sync_status reports CFDETR_ECAPACITY.
 */
CFDETR_API cfdetr_status cfdetr_fine_encode(cfdetr_ctx* ctx, const void* images, int32_t B,
                                 const int32_t* tok_desc, const int32_t* cu_seqlens,
                                 const float* x0_cache, float* y_mixed, void* hip_stream);

/*
 * The fine pass in the form the paper describes for A3 (Sec. III-B): the token sets of
 * the batch are padded to one length and go through the encoder as a dense batch; this
 * library masks the padded keys, so every real token gets exactly the result
 * cfdetr_fine_encode gives it.  A measurement mode: it shows what the variable-length
 * form saves.
 *   t_pad     tokens per frame after padding (host value), at least the longest frame of
 *             the batch and the coarse grid size; B * t_pad <= max_tokens_total
 *   y_padded  [B * t_pad, d] fp32 out: row f*t_pad + j is token j of frame f; rows of
 *             padding hold finite values without meaning
 * A frame longer than t_pad raises the sticky capacity flag (cfdetr_sync_status) and its
 * surplus tokens are ignored; a frame without tokens raises it too (the padded form has
 * no place for one) and its rows hold values without meaning.  Other arguments as in
 * cfdetr_fine_encode.
 */
CFDETR_API cfdetr_status cfdetr_fine_encode_padded(cfdetr_ctx* ctx, const void* images, int32_t B,
                                        const int32_t* tok_desc, const int32_t* cu_seqlens,
                                        const float* x0_cache, int32_t t_pad, float* y_padded,
                                        void* hip_stream);

/*
 * A1 -> A2 -> A3 in one call with no host synchronisation in between
 * (Sec. III-B, A1-A3).  Outputs are bit-identical to those of the three calls
 * above, but the encoder runs once: the B coarse grids and the B mixed token
 * sets form one variable-length batch of 2B sequences (multi-level batching,
 * A3, across the coarse and the fine subtask).  Arguments as in the three
 * calls above; level_counts may be NULL.
 */
CFDETR_API cfdetr_status cfdetr_multilevel_batch(cfdetr_ctx* ctx, const void* images, int32_t B,
                                      const int32_t* boxes, const uint8_t* tier,
                                      const int32_t* box_offsets, float* y_coarse,
                                      float* y_mixed, int32_t* tok_desc, int32_t* cu_seqlens,
                                      int32_t* level_counts, void* hip_stream);

/* ------------------------------------------------------------------------
 * Decoder (Sec. II-A: learned object queries attend to the encoded tokens of their frame
 * and come out as candidate boxes with a confidence).  The paper fixes no layer details;
 * this library's reading: n_queries learned vectors start every frame's queries; each of
 * the n_layers layers is pre-LN, x += SelfAttn(LN1 x); x += CrossAttn(LN2 x, tokens);
 * x += W2 GELU(W1 LN3 x); a final LayerNorm; the confidence is the logistic function of
 * one linear output, the box (cx, cy, w, h as fractions of the frame) the logistic
 * function of a three-layer perceptron with ReLU.  Widths, head count and FFN width are
 * the context's.  bf16 contexts only.
 * Weights (device pointers, matrices in bf16 bit patterns, vectors fp32, row-major,
 * stacked over layers like the encoder's):
 *   query_embed [Q, d] fp32
 *   ln1_g, ln1_b [L, d]; w_qkv [L, 3d, d]; b_qkv [L, 3d]; w_o [L, d, d]; b_o [L, d]
 *   ln2_g, ln2_b [L, d]; w_q [L, d, d]; b_q [L, d]; w_kv [L, 2d, d] (key rows, value
 *   rows); b_kv [L, 2d]; w_o2 [L, d, d]; b_o2 [L, d]
 *   ln3_g, ln3_b [L, d]; w_ff1 [L, F, d]; b_ff1 [L, F]; w_ff2 [L, d, F]; b_ff2 [L, d]
 *   lnf_g, lnf_b [d]; w_cls [1, d]; b_cls [1]; w_box1, w_box2 [d, d]; b_box1, b_box2 [d];
 *   w_box3 [4, d]; b_box3 [4]
 * ------------------------------------------------------------------------ */
typedef struct {
  int32_t n_queries; /* 1..1024 */
  int32_t n_layers;  /* >= 1   */
  const float* query_embed;
  const float *ln1_g, *ln1_b;
  const void* w_qkv;
  const float* b_qkv;
  const void* w_o;
  const float* b_o;
  const float *ln2_g, *ln2_b;
  const void* w_q;
  const float* b_q;
  const void* w_kv;
  const float* b_kv;
  const void* w_o2;
  const float* b_o2;
  const float *ln3_g, *ln3_b;
  const void* w_ff1;
  const float* b_ff1;
  const void* w_ff2;
  const float* b_ff2;
  const float *lnf_g, *lnf_b;
  const void* w_cls;
  const float* b_cls;
  const void* w_box1;
  const float* b_box1;
  const void* w_box2;
  const float* b_box2;
  const void* w_box3;
  const float* b_box3;
} cfdetr_decoder_weights;

/*
 * Gives the context a decoder: checks the weights and allocates the decoder's work space
 * (freed by cfdetr_destroy).  Once per context; the weights must outlive it and must not
 * change (re-ordered copies of some matrices are made here, as in cfdetr_create).
 */
CFDETR_API cfdetr_status cfdetr_decoder_attach(cfdetr_ctx* ctx, const cfdetr_decoder_weights* w);

/*
 * Object queries of every frame from its encoded tokens.
 *   memory      [T, d] fp32: encoder output (y_coarse or y_mixed), frame i at rows
 *               cu_seqlens[i] .. cu_seqlens[i+1]; T <= max_tokens_total
 *   cu_seqlens  [B+1] int32 (device), cu_seqlens[0] = 0, every frame at least one token.
 *               Checked on the device: a frame without tokens or a total above
 *               max_tokens_total makes the call read no token and the attention kernels do
 *               nothing, leaves `queries` undefined, and cfdetr_sync_status reports
 *               CFDETR_ECAPACITY.
 *   queries     [B, Q, 5] fp32 out: (cx, cy, w, h, c), the form cfdetr_propose_rois takes
 * Uses the context's encoder work space as scratch: a later encode call overwrites it,
 * and an encode call in flight on another stream must not overlap.
 */
CFDETR_API cfdetr_status cfdetr_decode(cfdetr_ctx* ctx, const float* memory,
                            const int32_t* cu_seqlens, int32_t B, float* queries,
                            void* hip_stream);

/* ------------------------------------------------------------------------
 * NPFP** scheduling decisions (Sec. IV).  Host memory only; no GPU work, no context,
 * no allocation.  Tasks are identified by index, index 0 has the highest priority,
 * deadlines equal periods.  At most 64 tasks.  WCETs come from tables measured
 * offline, as in the paper: coarse batches by batch size (c[x] for x subtasks, c[0]
 * unused), fine batches by the workload level of the largest member and the batch size
 * (row-major c[level * (max_size + 1) + size]).
 * ------------------------------------------------------------------------ */

typedef enum {
  CFDETR_POLICY_C = 0,    /* NPFP^C: coarse subtasks one by one, no fine subtasks      */
  CFDETR_POLICY_C_F = 1,  /* NPFP^CF                                                   */
  CFDETR_POLICY_BC_F = 2, /* NPFP^[C]F: coarse subtasks batched                        */
  CFDETR_POLICY_C_BF = 3, /* NPFP^C[F]: fine subtasks batched                          */
  CFDETR_POLICY_BC_BF = 4 /* NPFP^[C][F]                                               */
} cfdetr_policy;

typedef enum { CFDETR_SCHED_IDLE = 0, CFDETR_SCHED_COARSE = 1, CFDETR_SCHED_FINE = 2 } cfdetr_sched_action;

/*
 * Offline schedulability test of individually executed coarse subtasks (Lemma 1,
 * Eq. 3-4): R_i is the fixed point of R = C_i + B_i + sum_{h<i} ceil(R / T_h) C_h started
 * at C_i + B_i, B_i the longest coarse subtask of lower priority.
 *   period, c_coarse [n] in; response [n] out (infinity if the iteration passes T_i
 *   before it settles); *schedulable = 1 iff every R_i <= T_i.
 */
CFDETR_API cfdetr_status cfdetr_sched_response_times(int32_t n, const double* period,
                                          const double* c_coarse, double* response,
                                          int32_t* schedulable);

/*
 * Coarse batch assignment (Algo. 2): of the n_active active coarse subtasks, how many of
 * the highest-priority ones run now as one batch: the largest x >= 2 with
 * c_batch_by_size[x] <= next_release - t (Eq. 5), else 1 (0 if none is active).
 * Returns -1 on a bad argument.
 */
CFDETR_API int32_t cfdetr_sched_coarse_batch(int32_t n_active, double t, double next_release,
                                  const double* c_batch_by_size);

/*
 * Dynamic batch assignment of the active fine subtasks (Algo. 3, Lemma 3, Eq. 6).
 *   workload [n]  level of each subtask (0 = smallest), listed by priority
 *   deadline [n]  absolute deadlines
 *   t, next_coarse_release: now and the earliest future release of any task
 * Out: order [n]: the subtasks sorted by workload (stable); batch_end [n]: batch b is
 * order[batch_end[b-1] .. batch_end[b]) (batch_end[-1] = 0); *n_batches; dba [n+1]
 * (may be NULL): least total WCET of a schedulable partition of the first k sorted
 * subtasks, infinity if none.  A batch must end by every deadline in it and by
 * next_coarse_release.  If not all subtasks can be placed, the batches cover the longest
 * prefix of `order` that can.  Ties go to the shorter last batch.
 */
CFDETR_API cfdetr_status cfdetr_sched_fine_batches(int32_t n, const int32_t* workload,
                                        const double* deadline, double t,
                                        double next_coarse_release, const double* c_batch,
                                        int32_t n_levels, int32_t max_size, int32_t* order,
                                        int32_t* batch_end, int32_t* n_batches, double* dba);

/*
 * The decision at a scheduling instant (Algo. 1): coarse subtasks first (one, or a batch
 * under the [C] policies); else fine subtasks (one, if it ends before the next coarse
 * release, or the batches of cfdetr_sched_fine_batches under the [F] policies); else idle.
 *   active_coarse [n_coarse], active_fine [n_fine]: task indices in priority order;
 *   fine_workload, fine_deadline aligned with active_fine; next_release: earliest future
 *   release of any task.
 * Out: *kind; tasks [max(n_coarse, n_fine)]: the tasks to run, batch after batch;
 * batch_end / *n_batches as above (one batch for a coarse decision).
 */
CFDETR_API cfdetr_status cfdetr_sched_decide(cfdetr_policy policy, double t, int32_t n_coarse,
                                  const int32_t* active_coarse, int32_t n_fine,
                                  const int32_t* active_fine, const int32_t* fine_workload,
                                  const double* fine_deadline, double next_release,
                                  const double* c_coarse_by_size, const double* c_fine,
                                  int32_t n_levels, int32_t max_size,
                                  cfdetr_sched_action* kind, int32_t* tasks,
                                  int32_t* batch_end, int32_t* n_batches);

/*
 * Per-kernel timing with HIP events on the stream the kernels run on.
 * Between begin and end every launch is bracketed by an event pair (this costs
 * a few microseconds per launch, so timed throughput runs leave it off).
 * cfdetr_profile_end waits for the stream and fills two host arrays of
 * CFDETR_K_COUNT entries: summed milliseconds and launch counts per family.
 */
CFDETR_API cfdetr_status cfdetr_profile_begin(cfdetr_ctx* ctx);
CFDETR_API cfdetr_status cfdetr_profile_end(cfdetr_ctx* ctx, float* total_ms, int32_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* CFDETR_H */
