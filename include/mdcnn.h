/*
 * mdcnn.h -- C ABI of the MotionDeltaCNN hot path for AMD MI355X (gfx950).
 *
 * Sparse CNN inference of frame differences for moving-camera video: the state
 * of every layer lives in 2-D wrap-around ("spherical") ring buffers; per frame
 * and per layer the library computes the delta against the accumulated values,
 * truncates it into a per-pixel update mask, compacts the updated pixels, runs
 * the padded convolution on those pixels only and accumulates the result into
 * the next layer's ring buffer.
 *
 * Vocabulary.  A *site* is a tensor position that owns state: the network
 * input, every pre-activation tensor, every network output.  Per site:
 *   A  accumulated values (ring H x W)                       [Background: DeltaCNN]
 *   P  pending = truncated-values buffer, enlarged by the dilated border
 *      (ring (H+b0y+b1y) x (W+b0x+b1x))                      [Padded Convolutions]
 *   N/U/M per-frame bitmaps: newly unveiled / touched by a producer / updated
 *   L  compacted list of updated pixels (ascending view-linear index)
 * An *edge* is a linear operator between two sites: a k x k convolution
 * (optionally followed by nearest 2^n upsampling) or the identity (residual skip).
 *
 * Conventions.
 *  - All tensors are NHWC ("channels innermost"), storage dtype f32 or f16;
 *    arithmetic is always fp32 with one rounding per stored value.
 *  - Every `*_dev` pointer is DEVICE memory owned by the CALLER.  The library
 *    never allocates or frees device memory, never synchronises, and never reads
 *    device data back to the host: all work is enqueued on `stream`
 *    (a hipStream_t passed as void*; NULL = the default stream).
 *  - Handles (mdcnn_buffer*, mdcnn_net*) are small HOST objects owned by the
 *    library; destroy them with the matching call.
 *  - Errors are return codes.  Argument, shape and state errors are found before
 *    anything is enqueued or changed.  A HIP failure in the middle of a call
 *    (MDCNN_ERR_HIP) may leave launches enqueued: mdcnn_frame and its variants then
 *    mark every site of the network as never reset, so that the next camera shift
 *    re-initialises all buffers.  mdcnn_last_error() gives a thread-local
 *    description of the last failure.
 *  - One camera shift per frame: after mdcnn_shift_camera every non-terminal
 *    site must be passed through mdcnn_layer_forward (in topological order)
 *    before the next shift.  mdcnn_frame does exactly that.
 *  - Calls on the same buffers from several host threads or streams at once race.
 */
#ifndef MDCNN_H
#define MDCNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MDCNN_OK = 0,
    MDCNN_ERR_NULL = 1,    /* a required pointer is NULL                         */
    MDCNN_ERR_SHAPE = 2,   /* shapes / channels / borders of the operands disagree */
    MDCNN_ERR_DTYPE = 3,   /* unknown or mismatching storage dtype               */
    MDCNN_ERR_ALIGN = 4,   /* device pointer not aligned as documented           */
    MDCNN_ERR_SIZE = 5,    /* a byte count is too small / a size out of range    */
    MDCNN_ERR_STATE = 6,   /* call order violated (e.g. forward before first shift) */
    MDCNN_ERR_HIP = 7      /* a HIP launch failed; see mdcnn_last_error()        */
} mdcnn_status;

typedef enum { MDCNN_F32 = 0, MDCNN_F16 = 1 } mdcnn_dtype;
typedef enum { MDCNN_SITE_INPUT = 0, MDCNN_SITE_PREACT = 1, MDCNN_SITE_OUTPUT = 2 } mdcnn_site_kind;

/* Description of one site.  INPUT sites hold A only, OUTPUT sites hold P only. */
typedef struct {
    int H, W, C;              /* view extent in pixels of this site, channels           */
    int dtype;                /* mdcnn_dtype                                            */
    int kind;                 /* mdcnn_site_kind                                        */
    int border[4];            /* dilated border of P: before_y, after_y, before_x,      */
                              /* after_x (max over incoming edges, mdcnn_conv_border)   */
    int tile;                 /* pixels of this site per camera tile (total stride /    */
                              /* site stride)                    [Spherical Buffers]    */
    int relu;                 /* 1: f = ReLU, 0: f = identity                           */
    float theta;              /* truncation threshold on max-abs over channels, strict >*/
    const float* bias_dev;    /* C floats: sum of the biases of all producers, or NULL  */
    int origin_y, origin_x;   /* physical rotation of the rings (any value; results in  */
                              /* view order do not depend on it)                        */
    int pool_prev;            /* 1: destination of a max-pooling edge: the site also    */
                              /* keeps the previous pooling output of every view pixel  */
                              /* (ring H x W x C, PREACT sites only)                    */
    int crops;                /* 1: frames may cover a part of the view only            */
                              /* (mdcnn_set_crop); the site then keeps one more byte    */
                              /* per view pixel.  All sites of a network must agree.    */
    int truncation_free;      /* 1: the site never truncates and keeps NO pending ring: */
                              /* only A (half the state of the layer).  The output of   */
                              /* its producer is accumulated at once, A <- A + y, and   */
                              /* the change of the activation f(A + y) - f(A) is passed */
                              /* on wherever it is not zero (a newly unveiled pixel     */
                              /* starts from its bias and counts as updated).  For the  */
                              /* activation layers that do not follow a 3x3 convolution:*/
                              /* PREACT sites with ONE producer, a 1x1 convolution      */
                              /* without upsampling (any stride), hence no border; no   */
                              /* crops, no pooling.  theta is ignored (it is 0).        */
                              /* [Supplementary: Optimizing memory consumption]         */
} mdcnn_buffer_desc;

typedef struct mdcnn_buffer mdcnn_buffer;
typedef struct mdcnn_net mdcnn_net;

/* One edge.  Weights: w_dev[tap][cout][cin], tap = ky*k + kx, storage dtype of
 * the sites it joins, 16-byte aligned.  k == 0: identity edge (w_dev ignored,
 * stride 1, pad 0, up 0, Cin == Cout).  up > 0 requires k == 1, stride 1, pad 0.
 * w_packed_dev: NULL, or the copy of w_dev that mdcnn_pack_weights wrote (fp16,
 * Cin % 16 == 0); with it 3x3 stride-1 edges run on the faster matrix-core
 * kernel.  Both copies must stay valid and equal while the edge is in use. */
typedef struct {
    int k, stride, pad;
    int Cin, Cout;
    int up;                   /* log2 of the nearest-neighbour upsampling factor        */
    const void* w_dev;
    const void* w_packed_dev;
    int op;                   /* 0: convolution / identity as above.  1: k x k max pooling of */
                              /* the source's activations f(A) (in-view pixels of the window  */
                              /* only; weights ignored; Cin == Cout, up == 0, k >= 1): the    */
                              /* delta of an output pixel is taken against its previous       */
                              /* output, or against zero if the pixel is newly unveiled; the   */
                              /* destination must be a PREACT site with pool_prev = 1 and gets */
                              /* no border from this edge.  [Supplementary: Maximum Pooling]  */
} mdcnn_conv_desc;

/* Model preparation, once per edge: writes the weights of `edge` (w_dev, fp16,
 * Cin % 16 == 0, Cout % 32 == 0) to dst_dev in the order
 * [tap][cin/16][cout][16], in which the 32 couts x 16 cin operand of one
 * matrix-core instruction is 1 KiB of consecutive memory.  dst_dev: caller-owned
 * device memory, 16-byte aligned, dst_bytes == k*k*Cin*Cout*2 exactly.
 * Asynchronous on `stream`.  Errors: MDCNN_ERR_SHAPE for other shapes or dtypes. */
mdcnn_status mdcnn_pack_weights(const mdcnn_conv_desc* edge, int dtype, void* dst_dev, size_t dst_bytes,
                                void* stream);

/* Host-only helper.  The tile the halo-staged convolution kernel would cut an Hp x Wp padded window
 * into: the rectangle th x tw of at most max_pixels (1 .. 256) pixels whose footprint
 * (th + k - 1) x (tw + k - 1) has at most max_staged pixels and that covers the window with the
 * fewest tiles (ties: the smaller footprint); *tiles = ceil(Hp / th) * ceil(Wp / tw).
 * Errors: MDCNN_ERR_SHAPE if no rectangle fits, MDCNN_ERR_SIZE for arguments out of range.
 * [Padded Convolutions: a tile's outputs read the tile and a border of (k - 1) / 2 pixels around it] */
mdcnn_status mdcnn_conv_tiles(int Hp, int Wp, int k, int max_pixels, int max_staged, int* th, int* tw,
                              long long* tiles);

/* Host-only helper.  Width of the dilated border along one axis for a
 * convolution (k, stride, pad) from `in_extent` to `out_extent` pixels: how many
 * outputs before 0 / after out_extent-1 still read an in-view input.
 * 3x3 stride 1 pad 1 gives 1/1 (64 -> 66 outputs).        [Padded Convolutions] */
mdcnn_status mdcnn_conv_border(int k, int stride, int pad, int in_extent, int out_extent,
                               int* before, int* after);

/* Host-only.  Bytes of device memory a site needs (rings + per-frame scratch:
 * bitmaps, delta map, lists, counters).  Always a multiple of 256. */
mdcnn_status mdcnn_buffer_bytes(const mdcnn_buffer_desc* desc, size_t* bytes);

/* Wrap caller-owned device memory (256-byte aligned, >= mdcnn_buffer_bytes) as a
 * site.  Enqueues nothing; the memory may hold anything: the first
 * mdcnn_shift_camera performs a full reset.  The memory must stay valid until
 * mdcnn_destroy_buffer and must not be touched by the caller in between, except
 * through mdcnn_read_view / mdcnn_write_view.            [Spherical Buffers] */
mdcnn_status mdcnn_create_buffer(const mdcnn_buffer_desc* desc, void* dev_mem, size_t bytes,
                                 mdcnn_buffer** out);
mdcnn_status mdcnn_destroy_buffer(mdcnn_buffer* buf);

/* Move the camera by (dty, dtx) TILES for all `n` sites of one network at once
 * (pixel offset per site = tile offset x desc.tile).  Applies the buffer-manager
 * rule: a step against a direction in which the view has grown since the last
 * reset, a step of a whole view or more, or the very first call resets every
 * buffer (A = 0, P = bias, all pixels newly unveiled) and the frame is inferred
 * densely; otherwise only the pixels entering the padded window are initialised
 * (P = bias), pixels entering the view get A = 0 and are marked newly unveiled,
 * and stashed border values of pixels that move from the border into the view
 * are kept.  *did_full_reset (host, optional) is set to 0/1; it depends on the
 * shift history only.   [Buffer management; Dynamic Initialization; Supplementary:
 * Implicit bias application] */
mdcnn_status mdcnn_shift_camera(mdcnn_buffer* const* bufs, int n, int dty, int dtx,
                                void* stream, int* did_full_reset);

/* Cropped frames, host-only: from now on a frame covers tiles [ty0, ty0 + th) x
 * [tx0, tx0 + tw) of the view (tile offsets relative to the view as it lies after
 * the last mdcnn_shift_camera; they stay in force across later shifts until
 * changed; a new buffer starts with the whole view).  Site by site the crop is
 * that rectangle times desc.tile pixels.  Only pixels inside the crop are worked
 * on by mdcnn_layer_forward: of those, the ones no frame has covered since they
 * were allocated count as newly unveiled, and the ones a producer touched while
 * they lay outside earlier crops count as touched; a pixel a producer touches
 * outside the crop keeps the pending value and is remembered.  With the crop equal
 * to the view the results are those of a network without crops, bit for bit.
 * Errors: MDCNN_ERR_STATE if a buffer was created with crops == 0,
 * MDCNN_ERR_SHAPE if the rectangle is empty or leaves the view of a site.
 *                  [Spherical Buffers: cropped inputs, tile offset indices] */
mdcnn_status mdcnn_set_crop(mdcnn_buffer* const* bufs, int n, int ty0, int tx0, int th, int tw);

/* One layer of delta inference on site `in`:
 *   1. delta + truncation: INPUT site  d = frame - A;  PREACT site  d = f(A+P) - f(A)
 *      on the pixels a producer touched or that are newly unveiled;
 *      m = newly unveiled OR (forced mask given ? forced[p] : max_c |d_c| > theta);
 *      where m: A <- frame (resp. A+P), P <- 0, delta map <- d.
 *   2. compaction of m into the ascending list L (+ device-side count), and per
 *      edge the compute list = destination pixels (padded-window linear index,
 *      ascending) whose footprint holds an updated pixel.
 *   3. per edge, in the given order: y = conv(delta) on the compute list only,
 *      P_out <- P_out + y (border pixels included), U_out set.
 * `frame_dev`: H*W*C storage-dtype values in view order, INPUT sites only (else NULL).
 * `forced_mask_dev`: NULL, or H*W bytes (0/1) in view order replacing the
 * threshold test (with a forced mask on a PREACT site every in-view pixel is a
 * candidate).  `outs[i]` is the destination of `edges[i]`; OUTPUT sites take no
 * forward call.  On a site with a crop (mdcnn_set_crop) `frame_dev` and
 * `forced_mask_dev` have the crop's extent and order, and step 1 leaves the
 * pixels outside the crop alone.
 * Truncation-free sites (desc.truncation_free): as a DESTINATION, step 3 adds y to A
 * instead of P and produces the site's update mask and delta map right there, in the
 * arithmetic of steps 1 and 3 with theta 0 (y is rounded to the storage type as the
 * pending ring would hold it, on top of the bias for a newly unveiled pixel, then
 * added to A); the edge must be the site's only producer.  As the SOURCE `in`, step 1
 * is skipped (its mask and deltas exist already; a forced mask is an error,
 * MDCNN_ERR_STATE) and the call does steps 2 and 3.
 *                                  [Background: DeltaCNN; Padded Convolutions] */
mdcnn_status mdcnn_layer_forward(mdcnn_buffer* in, const void* frame_dev,
                                 const uint8_t* forced_mask_dev,
                                 const mdcnn_conv_desc* edges, mdcnn_buffer* const* outs,
                                 int n_edges, void* stream);

/* mdcnn_layer_forward for callers that cannot allocate device memory - code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc - and that created their sites from memory they
 * may not grow: the by-products of the call that only the library itself uses, i.e. the compacted list L
 * of `in`, the compute lists of the destinations and their per-segment counts and running sums, are
 * written to a buffer the library holds in a file-scope device array of 2 MiB (one per GPU the library
 * runs on, kept until the process ends) instead of the sites' own list regions.  Everything else - A, P,
 * delta maps, flags, the per-site counters of multiply-accumulates - is what mdcnn_layer_forward
 * produces, bit for bit; MDCNN_VIEW_LIST / MDCNN_VIEW_CLIST and the update / candidate / compute-list
 * entries of MDCNN_VIEW_STATS of the sites involved are NOT updated by this call.  The call allocates
 * nothing (no hipMalloc, no hipFree, no allocating library routine) and clears the part of the array it
 * uses with a fill kernel on `stream`.  All calls on one GPU share that array: calls that overlap in time
 * on one GPU (different streams or host threads) race.
 * Errors: those of mdcnn_layer_forward; MDCNN_ERR_SIZE if the lists of the call need more than the
 * 2 MiB (4 bytes per pixel of `in` and per padded-window pixel of every destination, plus 24 bytes per
 * 256 of them); MDCNN_ERR_HIP if the address of the array cannot be looked up. */
mdcnn_status mdcnn_layer_forward_noalloc(mdcnn_buffer* in, const void* frame_dev,
                                         const uint8_t* forced_mask_dev,
                                         const mdcnn_conv_desc* edges, mdcnn_buffer* const* outs,
                                         int n_edges, void* stream);

/* Network = sites in topological order + edges (edge i: sites[edge_src[i]] ->
 * sites[edge_dst[i]], edge_src non-decreasing).  Topology only; holds no device
 * memory.  Site 0 must be the only INPUT site. */
mdcnn_status mdcnn_net_create(mdcnn_buffer* const* sites, int n_sites,
                              const int* edge_src, const int* edge_dst,
                              const mdcnn_conv_desc* edges, int n_edges, mdcnn_net** out);
mdcnn_status mdcnn_net_destroy(mdcnn_net* net);

/* One frame: mdcnn_shift_camera, mdcnn_layer_forward over all non-terminal sites
 * in order, then the readout f(P) of every OUTPUT site in view order, written
 * back to back (site order) into out_dev (storage dtype; out_bytes must match
 * exactly).  `forced_mask_dev` applies to the input site only.  Results are
 * identical, bit for bit, to the same sequence of mdcnn_shift_camera /
 * mdcnn_layer_forward / mdcnn_read_view calls.                [Method, Fig. 3] */
mdcnn_status mdcnn_frame(mdcnn_net* net, const void* frame_dev, const uint8_t* forced_mask_dev,
                         int dty, int dtx, void* out_dev, size_t out_bytes, void* stream,
                         int* did_full_reset);

/* One cropped frame: mdcnn_shift_camera by (dty, dtx), mdcnn_set_crop(ty0, tx0, th,
 * tw), the forward calls, then the readout f(P) of every OUTPUT site over its crop,
 * in crop order (MDCNN_VIEW_CROP_OUT), back to back.  frame_dev / forced_mask_dev
 * cover the crop of the input site; out_bytes must equal the summed crop sizes.
 * All sites need crops == 1.  The crop stays in force afterwards. */
mdcnn_status mdcnn_frame_crop(mdcnn_net* net, const void* frame_dev, const uint8_t* forced_mask_dev,
                              int dty, int dtx, int ty0, int tx0, int th, int tw,
                              void* out_dev, size_t out_bytes, void* stream, int* did_full_reset);

/* Host-only.  The launch plan that mdcnn_frame follows for `net` when it may use
 * `streams` streams (1..4, or 0 for the library's own choice, see
 * MDCNN_OPT_STREAMS): one entry per kernel launch between the camera shift and the
 * readout, in launch order - per non-terminal site its delta launch, then one
 * launch per outgoing edge that gets one (a residual skip added by the delta kernel
 * gets none; a site without such edges gets one compaction launch).
 * stream_of[i]: stream of launch i (0 = the caller's); waits_of[2i], waits_of[2i+1]:
 * launches on other streams that launch i waits for, or -1 (launches on one stream
 * run in order anyway).  Both arrays are caller-owned with room for `cap` launches
 * (2 * cap ints for waits_of) and may be NULL; *n_launches and *n_streams (optional)
 * get the number of launches and of streams used.
 * Errors: MDCNN_ERR_SIZE if cap is too small or streams out of range. */
mdcnn_status mdcnn_frame_plan(mdcnn_net* net, int streams, int* stream_of, int* waits_of, int cap,
                              int* n_launches, int* n_streams);

/* The same for n_streams independent video streams in the same launches (the
 * paper fills the GPU with a batch of streams [Evaluation: batch size]).  Stream b
 * is nets[b]: all nets must have the same topology and the same site and edge
 * shapes, each its own buffers (weights may be shared); they keep their own
 * camera paths, masks and reset decisions.  All arrays are host arrays of
 * n_streams entries (1 <= n_streams <= 128; the streams share their launches in
 * groups of 16, group after group); frames_dev[b] / outs_dev[b] as in
 * mdcnn_frame, out_bytes per stream; forced_masks_dev may be NULL or hold NULL
 * entries; did_full_reset: n_streams ints or NULL.  The results of every stream
 * are identical, bit for bit, to those of mdcnn_frame on it alone.
 * Errors: MDCNN_ERR_SHAPE if the nets differ, MDCNN_ERR_STATE if two streams
 * share a net or buffers or a stream has a crop smaller than its view,
 * MDCNN_ERR_SIZE for n_streams out of range. */
mdcnn_status mdcnn_frame_batch(mdcnn_net* const* nets, int n_streams, const void* const* frames_dev,
                               const uint8_t* const* forced_masks_dev, const int* dty, const int* dtx,
                               void* const* outs_dev, size_t out_bytes, void* stream, int* did_full_reset);

/* mdcnn_frame_batch for cropped frames: stream b takes its frame with the crop
 * crops[4b .. 4b+3] = (ty0, tx0, th, tw) in tiles of the view, as mdcnn_frame_crop
 * does - every stream its own crop, camera path and output size (out_bytes[b] = the
 * summed crop sizes of the OUTPUT sites of stream b; frames_dev[b], its forced mask and
 * outs_dev[b] have that crop's extent).  All sites of all streams need crops == 1; the
 * crops stay in force afterwards.  The results of every stream are identical, bit for
 * bit, to those of mdcnn_frame_crop on it alone  [Supplementary: cropped frames;
 * Evaluation: batch size].
 * Errors: those of mdcnn_frame_batch and mdcnn_frame_crop, checked for all streams
 * before anything changes. */
mdcnn_status mdcnn_frame_batch_crop(mdcnn_net* const* nets, int n_streams,
                                    const void* const* frames_dev,
                                    const uint8_t* const* forced_masks_dev, const int* dty,
                                    const int* dtx, const int* crops, void* const* outs_dev,
                                    const size_t* out_bytes, void* stream, int* did_full_reset);

/* A run of n_frames consecutive frames of ONE video in one call, frame f being what
 * mdcnn_frame(net, frames_dev[f], forced_masks_dev[f], dty[f], dtx[f], outs_dev[f])
 * does: the frames are taken in order and every result - outputs and all state of the
 * sites - is identical, bit for bit, to n_frames calls of mdcnn_frame  [Method, Fig. 3].
 * What changes is when the launches run: several frames are in flight on `depth`
 * streams (stream 0 is the caller's, the others are the library's own, as for
 * MDCNN_OPT_STREAMS).  By default frame f as a whole goes to stream f % depth and
 * follows the frame before it at a distance of a few layers.  With MDCNN_OPT_PIPE_MODE
 * 0 the forward calls of the network are cut into `depth` runs of about equal cost
 * and run k of every frame goes to stream k, so that run k of frame f works next to
 * run k - 1 of frame f + 1.  Either way a frame touches a site only after the frame
 * before has finished with it: two launches on one site are either on one stream or
 * ordered by an event.  The initialisation of a camera shift is split by groups of
 * calls for this and done by spare blocks of the delta launches (MDCNN_OPT_PIPE_GROUP,
 * mdcnn_frames_plan).
 * These launches are bound by their latency, not by the size of the GPU, so overlapping
 * frames raises the frame rate of a single video the way a batch does for several; the
 * latency of a frame does not improve.
 * All arrays are host arrays of n_frames entries (1 <= n_frames <= 4096): frames_dev[f]
 * and outs_dev[f] device pointers as in mdcnn_frame (out_bytes each; the output buffers
 * must not overlap each other), forced_masks_dev NULL or with NULL entries,
 * did_full_reset n_frames ints or NULL.  depth: 1..4 streams; with 1 everything runs
 * on the caller's stream.  0: the library's default - 4 if a frame has at least 16
 * launches (mdcnn_frame_plan), else 1: on the benchmark networks with fewer launches
 * the events cost more than the overlap gains.
 * The caller's stream forks into the others at the start and waits for them at the end,
 * so the call as a whole stays in stream order; nothing is synchronised with the host.
 * With depth > 1 `stream` must not be capturing into a HIP graph (the fork into the
 * library's streams would be captured with it).
 * Errors: MDCNN_ERR_SIZE for n_frames, depth or out_bytes out of range, MDCNN_ERR_STATE
 * if outputs overlap or the network has a crop smaller than its view, MDCNN_ERR_NULL /
 * MDCNN_ERR_ALIGN as for mdcnn_frame (checked for all frames before anything runs). */
mdcnn_status mdcnn_frames(mdcnn_net* net, int n_frames, const void* const* frames_dev,
                          const uint8_t* const* forced_masks_dev, const int* dty, const int* dtx,
                          void* const* outs_dev, size_t out_bytes, int depth, void* stream,
                          int* did_full_reset);

/* mdcnn_frames for a batch of videos: n_frames consecutive frames of each of n_streams
 * independent videos (networks of equal topology and shapes with their own buffers,
 * camera paths, masks and reset decisions, as for mdcnn_frame_batch), with frames in
 * flight on `depth` streams as in mdcnn_frames.  One launch carries a forward call of
 * all videos (16 to a launch; with more, the whole run of the first 16 videos is
 * followed by that of the next 16 on the caller's stream), so a launch has n_streams
 * times the blocks and the frames in flight fill what is left of the GPU  [Evaluation:
 * batch sizes up to what the GPU holds; Method, Fig. 3].
 * Frame f of video b is what mdcnn_frame(nets[b], ...) does with entry [f * n_streams + b]
 * of frames_dev, forced_masks_dev (NULL or with NULL entries), dty, dtx, outs_dev
 * (out_bytes each, no two may overlap) and did_full_reset (NULL or n_frames * n_streams
 * ints): outputs and all state are identical, bit for bit, to those calls.
 * 1 <= n_streams <= 128, 1 <= n_frames <= 4096, depth as for mdcnn_frames.
 * Errors: as for mdcnn_frame_batch and mdcnn_frames, checked for all frames and videos
 * before anything runs; cropped frames are not supported (MDCNN_ERR_STATE if a network
 * has a crop smaller than its view). */
mdcnn_status mdcnn_frames_batch(mdcnn_net* const* nets, int n_streams, int n_frames,
                                const void* const* frames_dev,
                                const uint8_t* const* forced_masks_dev, const int* dty,
                                const int* dtx, void* const* outs_dev, size_t out_bytes,
                                int depth, void* stream, int* did_full_reset);

/* mdcnn_frames for cropped frames: frame f is what mdcnn_frame_crop does with the crop
 * (crops[4f .. 4f+3] = ty0, tx0, th, tw in tiles of the view); frames_dev[f], the forced
 * mask and outs_dev[f] have that crop's extent, out_bytes[f] the summed crop sizes of the
 * OUTPUT sites.  All sites need crops == 1; the last crop stays in force afterwards.
 * Everything else as for mdcnn_frames, results bit-identical to n_frames calls of
 * mdcnn_frame_crop.  Errors: also MDCNN_ERR_SHAPE for a crop that leaves the view; all
 * frames are checked before anything runs or changes. */
mdcnn_status mdcnn_frames_crop(mdcnn_net* net, int n_frames, const void* const* frames_dev,
                               const uint8_t* const* forced_masks_dev, const int* dty, const int* dtx,
                               const int* crops, void* const* outs_dev, const size_t* out_bytes,
                               int depth, void* stream, int* did_full_reset);

/* Host-only.  The plan mdcnn_frames follows for `net` on `depth` streams (0: default).
 * The forward calls of a frame (non-terminal sites in order) are numbered 0 ..
 * *n_calls - 1; the readout counts as call *n_calls.  stream_of_call[c] (c <= *n_calls):
 * the stream of call c in every frame (MDCNN_OPT_PIPE_MODE 0; -1 in mode 1, where frame
 * f is on stream f % depth).  Where the stream changes between two consecutive calls, the later
 * one waits for the earlier one of the same frame.  The calls are also cut into groups of
 * MDCNN_OPT_PIPE_GROUP calls: first_call[g]: first call of group g; group_of_site[i]: the
 * group the initialisation of site i belongs to (the first group with a launch that
 * touches the site); init_call[g]: the call whose delta launch carries that
 * initialisation in spare blocks (the last call of group g - 1, which does not touch
 * those sites; -1 for group 0, whose sites get a launch of their own ahead of call 0);
 * wait_call[g]: the call of the frame BEFORE that must have finished before that launch
 * starts (-1 for none) - the library waits for it with an event unless it is on the
 * same stream, where it comes earlier anyway.  The arrays are caller-owned with room for
 * cap_groups groups / cap_sites sites / cap_calls calls (*n_calls + 1 needed) and may
 * be NULL; *n_groups and *n_calls are optional.
 * Errors: MDCNN_ERR_SIZE if an array is too small or depth out of range. */
mdcnn_status mdcnn_frames_plan(mdcnn_net* net, int depth, int* first_call, int* wait_call,
                               int* init_call, int cap_groups, int* group_of_site, int cap_sites,
                               int* stream_of_call, int cap_calls, int* n_groups, int* n_calls);

/* Optional post-processing of the input update mask.  Writes, for the frame
 * `frame_dev` (not yet passed to a forward call), the mask that the threshold
 * test of the INPUT site `in` would give after these steps, as bytes 0/1 to be
 * handed to mdcnn_layer_forward / mdcnn_frame as the forced mask of that frame
 * (newly unveiled pixels are updated regardless):
 *   1. e(p) = max over channels of |frame - A|                [Background: DeltaCNN]
 *   2. with roi_dev (floats in [0, 1], e.g. the dilated previous result):
 *      e(p) *= sens_base + sens_gain * roi(p)   [Supplementary: ROI-focused sensing, 0.4 + 0.6 m]
 *   3. e is averaged over pool x pool cells (row by row, fp32) and the cells are
 *      compared with theta, strict >                                 [Optimizations]
 *   4. suppress = 1: a cell above the threshold with no other such cell among the
 *      3 x 3 cells around it is dropped                              [Optimizations]
 *   5. the cells cover their pixels and the mask is dilated by `dilate` pixels in
 *      every direction (10 spreads one pixel over 21 x 21), clipped to the frame
 *                                                    [Supplementary: first-layer dilation]
 * frame_dev, roi_dev (may be NULL) and mask_dev cover the site's crop (the view
 * without crops), row-major; mask_bytes must equal its pixel count.  All steps in
 * fp32.  Asynchronous on `stream`; reads A, changes no state.
 * Errors: MDCNN_ERR_SHAPE unless `in` is an INPUT site, pool is 1, 2, 4 or 8 and
 * divides both extents, 0 <= dilate <= 32, suppress is 0 or 1; MDCNN_ERR_STATE
 * before the first shift; MDCNN_ERR_SIZE for a wrong mask_bytes. */
typedef struct {
    float theta;
    float sens_base, sens_gain;
    int pool;
    int suppress;
    int dilate;
} mdcnn_mask_params;
mdcnn_status mdcnn_input_mask(const mdcnn_buffer* in, const void* frame_dev, const float* roi_dev,
                              const mdcnn_mask_params* prm, uint8_t* mask_dev, size_t mask_bytes,
                              void* stream);

/* mdcnn_frames with the mask front end: for frame f, after the camera shift, the library
 * runs mdcnn_input_mask(input site, frames_dev[f], roi_dev ? roi_dev[f] : NULL, prm) into
 * masks_dev[f] (mask_bytes = H*W of the input site each; n_frames caller-owned buffers that
 * must not overlap, kept as results) and forces that mask at the input site of frame f.
 * roi_dev may be NULL or hold NULL entries (maps that depend on earlier results of the same
 * call cannot be given: cut the video into shorter calls).  Everything else as for
 * mdcnn_frames; results bit-identical to mdcnn_shift_camera, mdcnn_input_mask,
 * mdcnn_layer_forward over all non-terminal sites and the readout, frame by frame.  Networks
 * without crops only.  Errors: those of mdcnn_frames and of mdcnn_input_mask, all
 * checked before anything runs; MDCNN_ERR_STATE also if two mask buffers overlap. */
mdcnn_status mdcnn_frames_masked(mdcnn_net* net, int n_frames, const void* const* frames_dev,
                                 const float* const* roi_dev, const mdcnn_mask_params* prm,
                                 uint8_t* const* masks_dev, size_t mask_bytes, const int* dty,
                                 const int* dtx, void* const* outs_dev, size_t out_bytes, int depth,
                                 void* stream, int* did_full_reset);

/* View-ordered access to a site's state (independent of the ring origin). */
typedef enum {
    MDCNN_VIEW_A = 0,        /* H*W*C storage dtype: accumulated values                     */
    MDCNN_VIEW_P = 1,        /* Hp*Wp*C storage dtype: pending values over the padded window */
                             /* (truncation-free sites have none: MDCNN_ERR_STATE)          */
    MDCNN_VIEW_DELTA = 2,    /* H*W*C storage dtype: delta map of the last forward (0 where not updated) */
    MDCNN_VIEW_FLAGS = 3,    /* H*W bytes: bit0 newly unveiled, bit1 touched, bit2 updated, */
                             /* bit3 visited by the last forward                            */
    MDCNN_VIEW_LIST = 4,     /* 1 + H*W int32: count, then the ascending list L             */
    MDCNN_VIEW_CLIST = 5,    /* 1 + Hp*Wp int32: count, then the compute list of the last   */
                             /* non-upsampling edge that produced into this site            */
    MDCNN_VIEW_STATS = 6,    /* 18 int32: [0] updated, [1] candidates, [2] compute-list      */
                             /* count of the last edge into this site; [8..17] five 64-bit  */
                             /* sums since creation: updated, candidates, multiply-         */
                             /* accumulates of the MFMA kernel into this site, compute-list */
                             /* entries, multiply-accumulates of the plain kernel           */
    MDCNN_VIEW_OUT = 7,      /* H*W*C storage dtype: f(P) over the view (readout)           */
    MDCNN_VIEW_POOL_PREV = 8,/* H*W*C storage dtype: previous pooling output (pool_prev sites) */
    MDCNN_VIEW_CROP_OUT = 9, /* h*w*C storage dtype: f(P) over the crop, crop order (read only) */
    MDCNN_VIEW_PENDING = 10  /* H*W bytes, sites with crops: bit0 no frame has covered the pixel */
                             /* since it was allocated, bit1 touched while outside the crops   */
} mdcnn_view;
mdcnn_status mdcnn_read_view(const mdcnn_buffer* buf, int what, void* dst_dev, size_t bytes,
                             void* stream);
/* Overwrite A, P, FLAGS, POOL_PREV or PENDING from view-ordered data (restoring a saved state). */
mdcnn_status mdcnn_write_view(mdcnn_buffer* buf, int what, const void* src_dev, size_t bytes,
                              void* stream);

/* Library options (process-wide, host-only). */
typedef enum {
    MDCNN_OPT_CONV_PATH = 0, /* 0 auto; fallbacks for testing: 1 plain FMA, 2 MFMA w/o LDS, */
                             /* 3 auto but never the packed-weights kernel                */
    MDCNN_OPT_PROFILE = 1,   /* 1: bracket every kernel launch with a pair of HIP events  */
    MDCNN_OPT_CONV_TILE = 2, /* tuning: 0 auto, 1..14 force a tile shape of the fp16 MFMA kernel; */
                             /* fp32 3x3 layers: 1 / 2 / 4 waves share the taps of a tile         */
    MDCNN_OPT_CONV_PIPE = 3, /* tuning: 0 auto, 1 / 2 prefetch depth of the MFMA kernel    */
    MDCNN_OPT_CONV_XCD = 4,  /* tuning: 1 (default) tie cout tiles to XCDs, 0 plain order  */
    MDCNN_OPT_CONV_KC = 5,   /* tuning: 0 auto, 64 cap the K step at 64 channels           */
    MDCNN_OPT_CONV_HALO = 6, /* tuning: 1 (default) packed-weights kernel where it applies,  */
                             /* 0 never, 2 with 32-cout tiles, 3 with tiles that are index  */
                             /* ranges of the padded window instead of rectangles, 4 with   */
                             /* rectangles also for windows of less than 4096 pixels (which */
                             /* take index ranges by default)                               */
    MDCNN_OPT_CONV_HALO_SUB = 7, /* 0 auto (by the tiles one video gives a launch), 1 / 2 / 4: tiles of a whole, */
                             /* half or quarter list segment (256 pixels) in that kernel; 1 is the faster choice for */
                             /* batches of many videos.  The split fixes the order of the sums: runs that are to  */
                             /* agree bit for bit need the same value                                              */
    MDCNN_OPT_FUSE_SKIP = 8, /* 1 (default): mdcnn_frame lets the delta kernel of a site add its   */
                             /* residual skip (identity edge) instead of a launch of its own; */
                             /* such an edge then adds nothing to the compute-list statistics  */
                             /* of its destination.  0: one launch per edge                  */
    MDCNN_OPT_PIPE_GROUP = 10, /* mdcnn_frames: forward calls per group of the frame pipeline (1..64): smaller */
                             /* groups let a frame follow the one before it more closely, at one more event   */
                             /* and wait per group and frame.  0 (default): about twenty groups per frame,    */
                             /* four calls per group at most                                                 */
    MDCNN_OPT_PIPE_THREADS = 12, /* mdcnn_frames: 1 (default) in mode 1, runs of at least 4 x depth frames are    */
                             /* issued by one host thread per stream (started and joined inside the call; a   */
                             /* frame is issued after the events it waits for have been recorded); 0: the     */
                             /* calling thread issues everything                                             */
    MDCNN_OPT_CONV_F32_MFMA = 13, /* 1 (default): fp32 layers with 16, 32 or 64 input and 16 or n x 32 output channels */
                             /* (1x1 or 3x3, no upsampling), and 3x3 stems with 3 input and n x 32 output    */
                             /* channels of either storage type, run on the matrix cores with the fp32       */
                             /* instruction; 0: plain FMA kernels (another summation order, same tolerance)  */
    MDCNN_OPT_PIPE_MODE = 11, /* mdcnn_frames: 1 (default) whole frames on streams, 0 runs of calls on streams */
    MDCNN_OPT_STREAMS = 9    /* 2..4: mdcnn_frame, mdcnn_frame_crop and mdcnn_frame_batch put       */
                             /* independent branches of the network on up to this many streams:     */
                             /* the caller's plus the library's own (per host thread, default     */
                             /* priority, created on first use).  The caller's stream forks into  */
                             /* them after the camera shift and waits for them before the readout, */
                             /* so the call stays in stream order; launches that write one site    */
                             /* keep their order, so the results do not change by a bit.  1: all   */
                             /* launches on the caller's stream.  0 (default): four streams if the */
                             /* network has parallel branches that shorten a frame by a fifth or   */
                             /* more (counted in launches, a wait for another stream as one), else */
                             /* the caller's stream only                                           */
} mdcnn_option;
mdcnn_status mdcnn_set_option(int option, int value);

/* Kernel classes reported by mdcnn_profile_read, in this order. */
typedef enum {
    MDCNN_K_SHIFT = 0, MDCNN_K_STEP1 = 1, MDCNN_K_LISTS = 2, MDCNN_K_CONV_MFMA = 3,
    MDCNN_K_CONV_PLAIN = 4, MDCNN_K_IDENTITY = 5, MDCNN_K_READOUT = 6, MDCNN_K_POOL = 7, MDCNN_K_COUNT = 8
} mdcnn_kernel_class;
/* Profiling mode only.  BLOCKS until the launches recorded since the last call
 * have finished, then returns per class the summed device time in milliseconds
 * and the number of launches (host arrays of n_classes == MDCNN_K_COUNT entries)
 * and forgets them.  Not thread-safe. */
mdcnn_status mdcnn_profile_read(int n_classes, double* ms, long long* launches);

/* Profiling mode only.  Like mdcnn_profile_read, but one entry per launch recorded since the
 * last read, in the order they were issued: its kernel class, the site whose forward call it
 * belongs to and the edge it executes (indices of mdcnn_net_create; -1: none, e.g. the delta
 * launch of a site has no edge, a launch outside mdcnn_frame has neither), and its device time
 * in microseconds.  Host arrays of `cap` entries; *n gets the number of launches (if it exceeds
 * cap nothing is forgotten and MDCNN_ERR_SIZE is returned).  BLOCKS until they have finished. */
mdcnn_status mdcnn_profile_read_launches(int cap, int* cls, int* site, int* edge, float* us, int* n);

/* Measurement helpers of the benchmark (not part of the path): what this machine reaches on a
 * plain copy and on back-to-back matrix-core instructions, to set beside the published peaks.
 * mdcnn_bench_copy: dst_dev <- src_dev, `bytes` (a multiple of 16, both 16-byte aligned), one
 * kernel, asynchronous on `stream`.  mdcnn_bench_mfma: `blocks` blocks of four waves issue
 * `iters` x 4 independent v_mfma_f32_32x32x16_f16 each; *flops (host, optional) gets the
 * floating-point operations of the launch; sink_dev: at least one float of device memory. */
mdcnn_status mdcnn_bench_copy(const void* src_dev, void* dst_dev, size_t bytes, void* stream);
mdcnn_status mdcnn_bench_mfma(int iters, int blocks, float* sink_dev, void* stream, double* flops);

const char* mdcnn_last_error(void);
const char* mdcnn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MDCNN_H */
