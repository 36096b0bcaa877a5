/*
 * hs.h -- C ABI of libhs: the per-frame hot path of N concurrent tool-tracking
 * application streams on one AMD MI355X (gfx950).
 *
 * The calls follow the problem statement of "Towards Deterministic End-to-end Latency
 * for Medical AI Systems in NVIDIA Holoscan" (arXiv 2402.04466):
 *   - an application is created once; its model is loaded at run time and one stream
 *     is created for the first operator and reused downstream (Section III-A);
 *   - it receives video frames one at a time and runs four stages per frame: format
 *     conversion, recurrent conv-net inference, tool-tracking postprocess, overlay of
 *     the result on the ORIGINAL frame (Section III-A);
 *   - every message is time-stamped on arrival at the first stage and on departure
 *     from the last; end-to-end latency is the difference (Section II-C, Section V-A);
 *   - each application gets an exclusive compute partition and is refused when its
 *     request exceeds what is free (Section IV-A "MPS Partition Creation" and
 *     "Admission Control").  Here the partition is a set of compute units (CUs) bound
 *     to the application's HIP streams with a CU mask, and the inference stages and
 *     the overlay stage can be given disjoint CU sets (the one-GPU analogue of the
 *     compute/graphics isolation of Section IV-B).
 *
 * Conventions
 *   - Pointers named d_* are DEVICE pointers (HIP global memory of the device given to
 *     hs_init); all others are host pointers.  No torch types cross this boundary.
 *   - All device memory is allocated and owned by the caller: the workspace given to
 *     hs_create_app, the input frames and the overlay outputs.  The library owns its
 *     HIP streams and events, a few KiB of pinned host memory per application, and
 *     its host threads.
 *   - Every call returns an hs_status; nothing throws or aborts across the boundary.
 *     hs_last_error() returns a thread-local description of the last failure.
 *   - Threading: one thread at a time may submit to a given application; any thread
 *     may poll it; different applications may be driven from different threads
 *     concurrently (the paper runs one process per application, Section V-B).
 */
#ifndef HS_H_
#define HS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hs_ctx hs_ctx; /* one per device, opaque */
typedef struct hs_app hs_app; /* one per application stream, opaque */
typedef struct hs_group hs_group; /* applications that share frames and one overlay, opaque */
typedef struct hs_mux hs_mux;     /* per-stream front of a batched application, opaque */

typedef enum {
  HS_OK = 0,
  HS_E_INVAL = -1,          /* NULL pointer, bad dimension, weight size mismatch       */
  HS_E_NOMEM = -2,          /* workspace too small / host allocation failed            */
  HS_E_OVERSUBSCRIBED = -3, /* admission control refused the partition                 */
  HS_E_QUEUE_FULL = -4,     /* all queue_depth slots hold unpolled or in-flight frames */
  HS_E_NOT_READY = -5,      /* no finished frame to deliver yet                        */
  HS_E_DEVICE = -6,         /* a HIP call failed; see hs_last_error()                  */
  HS_E_STATE = -7           /* call not allowed now (e.g. frames still in flight)      */
} hs_status;

typedef enum {
  /* 3->16 (stride 2) -> 32 (stride 2) -> 32 -> 8, all 3x3 pad 1, ReLU after the first
   * three layers, linear logits; stateless.  Logit map = net_h/4 x net_w/4.            */
  HS_NET_TINY4 = 1,
  /* ResNet-18-style backbone (7x7/2 stem + ReLU, 3x3/2 max-pool, 4 stages x 2 basic
   * blocks, widths 64/128/256/512, 1x1/2 projection shortcuts, no normalisation, no
   * bias) + one ConvLSTM cell (512+256 -> 4x256, 3x3, gate order i,f,g,o, state carried
   * across frames) + 1x1 head 256 -> 8.  Logit map = ceil(net/32) per axis.            */
  HS_NET_RESNET18_CONVLSTM = 2
} hs_net_kind;

#define HS_NUM_TOOLS 8      /* output channels of either network = tool classes        */
#define HS_MAX_CU_WORDS 8   /* CU masks are bit sets of up to 256 CUs, 32 per word      */

/* Application description (read by hs_query_workspace and hs_create_app; copied). */
typedef struct {
  int frame_w, frame_h;     /* input video frame, pixels                                */
  size_t frame_pitch;       /* bytes between frame rows, >= 3*frame_w; rows are RGBRGB.. */
  int net_w, net_h;         /* size the frame is resized to for the network              */
  int net_fp32_input;       /* 1: stage 1 also stores the converted tensor as planar fp32 */
  float mean, std;          /* normalisation: (v/255 - mean) / std                       */
  float threshold;          /* heat-map threshold in (0,1), compared strictly (>)        */
  float alpha;              /* overlay opacity in [0,1], quantised to 1/256 steps        */
  int net;                  /* hs_net_kind                                               */
  const float* weights;     /* HOST fp32 blob: layers in network order, each             */
                            /* [Cout][Cin][kh][kw]; copied and repacked to fp16 at create */
  size_t weight_floats;     /* number of floats in the blob; must match the network      */
  uint8_t palette[HS_NUM_TOOLS][3]; /* overlay colour per tool channel, RGB              */
  int queue_depth;          /* frames (batches) that may be in flight or unpolled, 1..64. */
                            /* With an even depth consecutive frames run in two lanes (own */
                            /* activation buffers and stream) and overlap on the GPU; only */
                            /* the recurrent cell chains them. Results do not depend on it. */
  int batch;                /* streams served by this application, 1..16. With batch > 1  */
                            /* the streams share one weight copy and every submit carries */
                            /* one frame of each stream; stages 1, 3, 4 run per stream,   */
                            /* the network runs once over the whole batch (ConvLSTM state */
                            /* per stream). Use hs_submit_batch / hs_poll_batch then.     */
  /* Annotation layer of stage 4 (paper Section III-A: the visualisation draws the segmented
   * tools and their text labels).  With annotate != 0, for every tool k whose present flag
   * is set, in increasing k and opaque in palette[k], on top of the blended masks:
   * a cross-hair centred on the argmax cell's footprint, cx = ((2*ax+1)*frame_w)/(2*map_w),
   * cy likewise (arms marker_arm pixels long, 2*marker_half+1 thick), and the label 'T'<k>
   * (glyphs of 5 x 7 cells, glyph_scale pixels per cell, second glyph 6*glyph_scale to the
   * right, label origin (cx + marker_arm + 2, cy - 7*glyph_scale - 2)); clipped to the frame. */
  int annotate;             /* 0: masks only                                             */
  int marker_arm;           /* 0..64                                                     */
  int marker_half;          /* 0..8                                                      */
  int glyph_scale;          /* 1..8                                                      */
  uint8_t glyphs[9][7];     /* 'T','0'..'7': 7 rows of 5-bit masks, bit 4 = left column  */
  void* d_workspace;        /* DEVICE memory owned by the caller, 256-byte aligned       */
  size_t workspace_bytes;   /* >= hs_query_workspace(); plays the role of the per-client  */
                            /* device-memory limit of the paper's partitions              */
} hs_app_desc;

/* What stage 3 found for one frame, plus the frame's time stamps. All times are
 * CLOCK_MONOTONIC nanoseconds. t_submit_ns is taken on entry to hs_submit_frame
 * (arrival at the first stage). t_overlay_done_ns is taken by the library's completion
 * thread when the overlay kernel's completion event fires (departure from the last
 * stage) -- independent of when the caller polls; t_observed_ns is the poll time;
 * t_enqueued_ns is when hs_submit_frame had handed all work to the GPU queues (host
 * launch cost = t_enqueued_ns - t_submit_ns).
 * The three intermediate stamps are t_overlay_done_ns minus the GPU-event time between
 * that stage's end and the overlay's end.  End-to-end latency = t_overlay_done_ns -
 * t_submit_ns (Section II-C).
 *
 * Device pointers alias the queue slot the frame was given inside the application's
 * workspace and stay valid until queue_depth further frames have been submitted to the
 * same application.
 *   d_net_input     fp16, pixel-interleaved with 4 channels per pixel (R,G,B,0),
 *                   net_h rows of net_w pixels, row pitch net_input_pitch_bytes
 *   d_net_input_f32 fp32 planar [3][net_h][net_w], or NULL unless net_fp32_input
 *   d_logits        fp32 planar [8][map_h][map_w]
 *   d_heat          fp32 planar [8][map_h][map_w] = sigmoid(logits)
 *   d_mask          uint8 planar [8][map_h][map_w] in {0,1}
 *   d_overlay       the caller's d_overlay_out for this frame
 */
typedef struct {
  uint64_t frame_id;
  uint64_t t_submit_ns, t_enqueued_ns, t_pre_done_ns, t_infer_done_ns, t_post_done_ns,
      t_overlay_done_ns, t_observed_ns;
  int32_t argmax_idx[HS_NUM_TOOLS]; /* row-major index y*map_w+x of the channel maximum,  */
                                    /* lowest index among equal maxima                    */
  uint8_t present[HS_NUM_TOOLS];    /* 1 if the channel maximum exceeds the threshold     */
  float peak[HS_NUM_TOOLS];         /* sigmoid of the channel maximum                     */
  int map_w, map_h;
  size_t net_input_pitch_bytes;
  const void* d_overlay;
  const void* d_mask;
  const void* d_heat;
  const void* d_logits;
  const void* d_net_input;
  const void* d_net_input_f32;
} hs_result;

/* Latency determinism metrics of Section V-A, in the unit of the input. */
typedef struct {
  uint64_t n;      /* samples left after trimming                                        */
  double mean, max, std; /* std: population standard deviation                           */
  double p50, p99;
  double tail;     /* 100th - 95th percentile                                            */
  double flatness; /* 90th - 10th percentile                                             */
} hs_latency_metrics;

/* Aggregated kernel timing of one application (see hs_set_kernel_timing). */
typedef struct {
  char name[48];      /* kernel family, e.g. "conv_mfma", "resize_norm", "overlay"       */
  uint64_t launches;  /* launches timed since the last reset                             */
  double total_ms;    /* sum of HIP-event elapsed time over those launches               */
  double flops;       /* algorithmic flops of those launches (0 for byte-bound kernels)   */
  double bytes;       /* algorithmic bytes of those launches (0 for flop-bound kernels)   */
} hs_kernel_time;

/* ---- context ------------------------------------------------------------------- */

/* Bind a context to HIP device `device` (makes it current for the calling thread).
 * HS_E_DEVICE if there is no such GPU or it is not a gfx950 part. */
hs_status hs_init(int device, hs_ctx** out);
/* Destroys the context. All its applications must have been destroyed (HS_E_STATE). */
hs_status hs_shutdown(hs_ctx* ctx);
/* Number of CUs of the context's device (256 on MI355X). */
hs_status hs_device_cus(hs_ctx* ctx, int* n_cus);

/* ---- application life cycle (Section III-A: model loaded at run time, stream created
 *      once and reused by the later stages) ---------------------------------------- */

/* Device bytes hs_create_app needs for this description (weights in fp16, activation
 * and state buffers, queue_depth result slots). Pure host computation. */
hs_status hs_query_workspace(const hs_app_desc* desc, size_t* bytes);
/* Validates the description, repacks and uploads the weights into the workspace, zeroes
 * the recurrent state, creates the application's two HIP streams (inference stages;
 * overlay stage), its events and its completion thread. Synchronous. The application
 * starts unpartitioned (all CUs). */
hs_status hs_create_app(hs_ctx* ctx, const hs_app_desc* desc, hs_app** out);
/* Waits for in-flight frames, stops the completion thread, releases streams, events and
 * claimed CUs. The workspace returns to the caller. */
hs_status hs_destroy_app(hs_app* app);
/* Zero the ConvLSTM state (h, c). HS_E_STATE while frames are in flight. */
hs_status hs_reset_state(hs_app* app);
/* Copy the ConvLSTM state of the last completed frame to HOST buffers, as fp32 planar
 * [256][map_h][map_w] each (either may be NULL). HS_E_STATE while frames are in flight,
 * HS_E_INVAL for a stateless network. For tests and for checkpointing a stream. */
hs_status hs_get_state(hs_app* app, int stream, float* h_out, float* c_out);
/* Copy the backbone's output for the last completed frame (the ConvLSTM cell's input x_t)
 * to a HOST buffer as fp32 planar [512][map_h][map_w]. Same status rules as hs_get_state.
 * Lets a test check the recurrent cell in isolation. `stream` < batch in both calls. */
hs_status hs_get_features(hs_app* app, int stream, float* x_out);

/* ---- spatial partition + admission control (Section IV-A) ------------------------- */

/* Bind the application's inference stream (stages 1-3) and overlay stream (stage 4) to
 * CU sets. Masks are bit sets, bit i of word i/32 = CU i, n_words <= HS_MAX_CU_WORDS.
 * The two masks may be disjoint (compute / visualisation isolation: two streams, i.e. two
 * hardware queues) or equal (one stream carries all four stages).  The device executes at
 * most four hardware queues truly concurrently; queues beyond that share a pipe and their
 * frames serialise, so more than two partitioned applications should use equal masks.
 * Admission control: refused with HS_E_OVERSUBSCRIBED, changing nothing, if a mask is
 * empty, names a CU the device does not have, or intersects CUs claimed by another
 * application of the context. On MI355X CU i belongs to XCD i mod 8 and every mask must
 * contain at least one CU of each XCD (HS_E_INVAL otherwise): build masks from whole groups
 * of 8 consecutive CUs. Passing NULL for both masks releases the claim and
 * returns the application to the unpartitioned state (all CUs, claims nothing).
 * HS_E_STATE while frames are in flight. */
hs_status hs_set_partition(hs_app* app, const uint32_t* cu_mask_infer,
                           const uint32_t* cu_mask_overlay, int n_words);
/* The admission predicate alone, on host data (no GPU needed): would a request for
 * req_infer | req_overlay be admitted given the CUs already claimed by others?
 * Returns HS_OK or HS_E_OVERSUBSCRIBED / HS_E_INVAL exactly as hs_set_partition would (it is
 * the same function): HS_E_OVERSUBSCRIBED for an empty mask, a CU >= device_cus or a claimed
 * CU; HS_E_INVAL for bad arguments or a mask without a CU on each of the device_cus / 32 XCDs. */
hs_status hs_admission_check(const uint32_t* claimed_by_others, const uint32_t* req_infer,
                             const uint32_t* req_overlay, int n_words, int device_cus);

/* ---- per-frame hot path (Section III-A) ------------------------------------------- */

/* Enqueue the four stages for one frame and return without waiting.
 *   d_frame       device, frame_h rows of frame_pitch bytes, RGB uint8; read by stage 1
 *                 and again by stage 4; must stay untouched until the result is polled
 *   d_overlay_out device, same shape and pitch as d_frame; written by stage 4; must not
 *                 alias d_frame
 * Frames of one application are processed strictly in submit order (the recurrent
 * state of frame t feeds frame t+1). HS_E_QUEUE_FULL (frame NOT enqueued) when
 * queue_depth frames are in flight or unpolled.  If a HIP call fails after part of the frame
 * has been handed to the GPU (HS_E_DEVICE), the recurrent state may already have been advanced
 * by a frame that is never delivered: the application is unusable from then on, every later
 * submit returns HS_E_DEVICE, and it must be destroyed.  The same holds for every member of a
 * group when hs_submit_group fails that way. */
hs_status hs_submit_frame(hs_app* app, const uint8_t* d_frame, uint8_t* d_overlay_out,
                          uint64_t frame_id);
/* hs_submit_frame for callers that cannot allocate device memory or let the library touch an
 * allocator while they run: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same results bit for bit, same status codes; the call
 * allocates nothing, neither on the device nor (on its success path) on the host.  The one
 * scratch buffer of the hot path, the fp32 partial sums of the convolutions that are split
 * along K, is taken from a fixed 8 MiB device array inside the library (one copy per GPU, held
 * until the process ends) instead of the application's workspace; kernels are always launched
 * one by one (never as a HIP graph).  The 1920x1080 -> 854x480 network needs 6.6 MB of it.
 *   HS_E_NOMEM  a frame of this application needs more scratch than the array holds
 *               (hs_last_error() names both sizes); nothing is enqueued
 *   HS_E_STATE  batched or grouped application, kernel timing switched on, or a frame of this
 *               application still in flight (the call takes one frame at a time)
 * Every call on a GPU shares that GPU's array, which holds whatever the last frame left in it
 * (every value a frame reads it has written before, so nothing needs clearing).  Frames of
 * DIFFERENT applications submitted through this call must not be in flight together on one GPU:
 * they race on the array and the library does not detect it.  Frames submitted through the
 * other calls are not affected. */
hs_status hs_submit_frame_static_scratch(hs_app* app, const uint8_t* d_frame,
                                         uint8_t* d_overlay_out, uint64_t frame_id);
/* Deliver the oldest finished, not yet delivered frame (submit order). Non-blocking:
 * HS_E_NOT_READY if none has finished. Frees that frame's queue slot. */
hs_status hs_poll_result(hs_app* app, hs_result* out);
/* As hs_poll_result, but sleeps until a frame has finished or timeout_ns elapsed
 * (HS_E_NOT_READY on time-out). */
hs_status hs_wait_result(hs_app* app, hs_result* out, uint64_t timeout_ns);

/* Batched applications (desc.batch = B > 1): one frame of each of the B streams per call.
 * d_frames / d_overlay_outs are HOST arrays of B device pointers (same rules per frame as
 * hs_submit_frame). The B frames share the time stamps of the call; results come back as B
 * consecutive hs_result entries (stream order) written to out[0..B-1]. The single-frame
 * calls above return HS_E_STATE on a batched application; with B = 1 both forms work. */
hs_status hs_submit_batch(hs_app* app, const uint8_t* const* d_frames,
                          uint8_t* const* d_overlay_outs, uint64_t frame_id);
hs_status hs_poll_batch(hs_app* app, hs_result* out);
hs_status hs_wait_batch(hs_app* app, hs_result* out, uint64_t timeout_ns);
/* As hs_submit_batch (also for batch = 1) when the frames are still being produced on one of the
 * caller's own HIP streams: hip_event_frames_ready is a hipEvent_t the caller recorded on that
 * stream after the last write to the frames; stage 1 is ordered behind it on the GPU, the call
 * itself does not wait.  NULL: no dependency.  The stage-4 read of the frames is ordered behind
 * stage 1 anyway.  t_submit_ns is still the time of the call. */
hs_status hs_submit_batch_after(hs_app* app, const uint8_t* const* d_frames,
                                uint8_t* const* d_overlay_outs, uint64_t frame_id,
                                void* hip_event_frames_ready);

/* ---- multi-network applications (Section III-B) ------------------------------------- */

/* The paper's second application runs three networks on every frame, each behind its own
 * format converter, in parallel GPU streams, and one visualisation renders the aggregated
 * layers over the original frame.  Here: a group of 1..HS_MAX_GROUP applications of one
 * context (each created with hs_create_app: own network, network input size, threshold,
 * palette, alpha, annotation settings, workspace; batch 1; identical frame_w, frame_h and
 * frame_pitch).  hs_submit_group hands ONE frame to all members: each runs stages 1-3 on its
 * own stream(s), side by side on the GPU (member 0's work is enqueued by the calling thread,
 * every other member's by a thread of its own, as the paper's inference operator spawns one CPU
 * thread per parallel inference), and a single stage-4 launch, on member 0's overlay
 * stream after every member's stage 3, draws the members' layers in member order -- a
 * member's mask blend, then its annotations, each layer over the picture the previous one
 * left -- into d_overlay_out (the frame is read once and written once).
 * Results arrive as n_members consecutive hs_result entries (member order) once every member
 * has finished the frame; all carry the same t_submit_ns and d_overlay, and t_overlay_done_ns
 * is stamped by each member's completion thread when the shared overlay launch completes.
 * While grouped, members are driven only through the group: their own submit / poll / wait /
 * destroy calls return HS_E_STATE; hs_set_partition, hs_reset_state, hs_get_state and the
 * launch-mode and timing calls still address single members (the shared overlay launch is
 * accounted to member 0).  One thread at a time submits to a group, one thread at a time polls.
 *
 * hs_create_group: HS_E_INVAL for NULL / foreign / repeated / batched members or differing
 * frame geometry, HS_E_STATE if a member is already grouped or has frames in flight or
 * unpolled.  The members array is copied.
 * hs_destroy_group: waits for in-flight frames, then releases the members (results not yet
 * polled stay available through the members' own poll calls). */
#define HS_MAX_GROUP 4
hs_status hs_create_group(hs_ctx* ctx, hs_app* const* members, int n_members, hs_group** out);
hs_status hs_destroy_group(hs_group* group);
/* Same frame rules as hs_submit_frame. HS_E_QUEUE_FULL (nothing enqueued for any member) when
 * a member has no free slot. */
hs_status hs_submit_group(hs_group* group, const uint8_t* d_frame, uint8_t* d_overlay_out,
                          uint64_t frame_id);
/* out[0 .. n_members-1]. Non-blocking / blocking as hs_poll_result / hs_wait_result. */
hs_status hs_poll_group(hs_group* group, hs_result* out);
hs_status hs_wait_group(hs_group* group, hs_result* out, uint64_t timeout_ns);

/* How hs_submit_frame hands stages 1-3 to the GPU: kernel by kernel (default), or as one
 * pre-built HIP graph per queue slot (one launch call per frame instead of ~35: a third less
 * host time per frame, but the GPU sees the first kernel only once the whole graph has been
 * handed over, which measured 20-30 us more latency per frame in every configuration).
 * Results are identical. Kernel timing (below) always uses the kernel-by-kernel path.
 * HS_E_STATE while frames are in flight. */
#define HS_LAUNCH_GRAPH 0
#define HS_LAUNCH_EAGER 1
hs_status hs_set_launch_mode(hs_app* app, int mode);

/* ---- measurement ------------------------------------------------------------------ */

/* Section V-A / Section VI metrics of n latencies. trim != 0 first discards
 * min(10, n/6) samples from each end in the given (arrival) order, the paper's warm-up
 * and cool-down rule scaled to short runs. Percentiles interpolate linearly between
 * closest ranks. HS_E_INVAL if nothing is left. Pure host computation. */
hs_status hs_latency_metrics_compute(const double* latencies, size_t n, int trim,
                                     hs_latency_metrics* out);
/* Two-sided Mann-Whitney U comparison of two latency samples (paper, appendix "Additional
 * Evaluation": two configurations differ when |Z| > 1.96 at significance level 0.05).
 * u = number of pairs (a_i, b_j) with a_i > b_j plus half the ties; z = normal approximation
 * with tie-corrected variance and 0.5 continuity correction, 0 when the variance vanishes.
 * Pure host computation on HOST arrays; HS_E_INVAL if an array is NULL or empty. */
typedef struct {
  double u;          /* U statistic of sample a                                           */
  double z;          /* > 0: a tends to be larger than b                                  */
  int significant;   /* |z| > 1.96                                                        */
} hs_mwu;
hs_status hs_mann_whitney_u(const double* a, size_t na, const double* b, size_t nb, hs_mwu* out);

/* Pin the application's completion thread (the one that observes the end of a frame and
 * stamps its departure) to one CPU core, cpu = -1 lifts the pin (paper Section IV-C, CPU
 * affinity). The caller pins its own submitting thread with sched_setaffinity. For a member
 * of a group (call it after hs_create_group) the thread that enqueues this member's stages is
 * pinned to the same core.
 * HS_E_INVAL if the core does not exist or the operating system refuses. */
hs_status hs_set_cpu_affinity(hs_app* app, int cpu);

/* enable != 0: bracket every kernel launch of this application with HIP events on the
 * launching stream and accumulate elapsed time per kernel family (adds event overhead;
 * meant for roofline measurements, off by default). Switching resets the accumulators.
 * HS_E_STATE while frames are in flight. */
hs_status hs_set_kernel_timing(hs_app* app, int enable);
/* Copy up to max_entries accumulated entries; *n_entries receives the count available.
 * Collects finished events first. HS_E_STATE while frames are in flight. */
hs_status hs_get_kernel_times(hs_app* app, hs_kernel_time* entries, int max_entries,
                              int* n_entries);

/* Plain device-to-device streaming copy of `bytes` (multiple of 16, 16-byte aligned, no
 * overlap) on the default stream, synchronous. Its only purpose is measurement: it is the
 * kernel of known traffic against which hardware byte counters (rocprofv3 FETCH_SIZE /
 * WRITE_SIZE) are scaled. */
hs_status hs_device_copy(hs_ctx* ctx, void* d_dst, const void* d_src, size_t bytes);

/* ---- batched application fed stream by stream ---------------------------------------- */

/* A batched application (desc.batch = B) takes one frame of every stream per call of
 * hs_submit_batch.  Independent sources do not arrive together: the mux lets stream j hand
 * over its frame on its own (hs_mux_submit, from any thread; arrival is stamped then), submits
 * the batch to the application when the last of the B frames has arrived, and lets every
 * stream collect its own result (hs_mux_poll / hs_mux_wait: the hs_result of that stream, with
 * t_submit_ns = the stream's own arrival and frame_id = the id the stream gave, so that
 * t_overlay_done_ns - t_submit_ns includes the wait for the rest of the batch).
 * A stream whose previous frame still waits for its batch gets HS_E_QUEUE_FULL, and so does the
 * stream that would complete a batch while the application's queue is full (its frame is not
 * taken, the others keep waiting).  While a mux exists the application is driven only through
 * it.  The calls are thread-safe among themselves.  hs_create_mux: HS_E_INVAL unless `batch`
 * equals the application's batch, HS_E_STATE for a member of a group. */
hs_status hs_create_mux(hs_app* app, int batch, hs_mux** out);
hs_status hs_destroy_mux(hs_mux* mux);
hs_status hs_mux_submit(hs_mux* mux, int stream, const uint8_t* d_frame, uint8_t* d_overlay_out,
                        uint64_t frame_id);
hs_status hs_mux_poll(hs_mux* mux, int stream, hs_result* out);
hs_status hs_mux_wait(hs_mux* mux, int stream, hs_result* out, uint64_t timeout_ns);

/* ---- native stream driver --------------------------------------------------------- */

/* One source of frames: an application (batch >= 1), a group or one stream of a mux, with the
 * device buffers it cycles through.  d_frames / d_outs are HOST arrays of n_frames * batch /
 * n_outs * batch device pointers; frame k submits entries (k % n_frames) * batch .. + batch - 1 as input and
 * (k % n_outs) * batch .. as overlay output (n_outs >= queue_depth keeps an output untouched
 * until its result has been collected).  frame_id = k. */
typedef struct {
  hs_app* app;               /* ignored when group or mux is given                         */
  hs_group* group;           /* a multi-network application, batch must be 1               */
  hs_mux* mux;               /* one stream (mux_stream) of a batched application behind a   */
  int mux_stream;            /* mux; batch and results_per_frame must be 1                  */
  const uint8_t* const* d_frames;
  uint8_t* const* d_outs;
  int n_frames, n_outs, batch;
  int results_per_frame;     /* batch, or the group's member count                         */
  int cpu;                   /* core the submitting thread pins itself to, -1: none        */
} hs_feed;
/* Drives n_feeds sources concurrently, one submitting thread each (the paper runs one
 * process per application, Section V-B), for n_frames frames per source, and returns when
 * every result has been collected.  fps > 0: frame k of every source is submitted at
 * t0 + k / fps (absolute deadlines, clock_nanosleep on CLOCK_MONOTONIC); a frame that finds
 * its queue full is dropped and counted.  fps == 0: back to back, as fast as the queues take
 * the frames (nothing is dropped: a full queue is waited on).
 * results[i] receives the collected frames of source i in order, results_per_frame entries
 * each (HOST array of n_frames * results_per_frame entries; with drops the tail stays
 * unwritten); dropped[i] (may be NULL) the number of dropped frames; lateness_ns[i] (array or
 * the whole argument may be NULL) how long after its deadline frame k was submitted;
 * *elapsed_s (may be NULL) the wall time from starting the submitting threads to the
 * collection of the last result, i.e. with all GPU work of the run complete.
 * The sources must not be used by other threads meanwhile.  First failing status of any
 * source is returned after all threads have ended. */
hs_status hs_run_feeds(const hs_feed* feeds, int n_feeds, double fps, int n_frames,
                       hs_result* const* results, int* dropped, int64_t* const* lateness_ns,
                       double* elapsed_s);

/* The same plain copy, `repeats` times back to back on the application's overlay stream, i.e.
 * under the CU mask the application's partition gives that stream (all CUs when it is not
 * partitioned); *seconds_per_copy = GPU time between events around the repeats / repeats (one
 * untimed copy first).  It measures what the partition's CUs can pull: the denominator for the
 * byte-bound kernels of a partitioned application.  Same argument rules as hs_device_copy;
 * HS_E_STATE while frames are in flight. */
hs_status hs_partition_copy(hs_app* app, void* d_dst, const void* d_src, size_t bytes,
                            int repeats, double* seconds_per_copy);

/* Thread-local, never NULL; valid until the next failing call on this thread. */
const char* hs_last_error(void);
/* Library version string. */
const char* hs_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HS_H_ */
