/*
 * libocto - the data-parallel hot path of a cascaded video-analytics serving
 * pipeline on one AMD MI355X (gfx950).
 *
 * The serving problem follows OctopInf (arXiv 2502.01277): a pipeline is a DAG of
 * DNN models (Sec. II), each served with a batch size and an execution slot
 * [bz, d, g, t]; all queries of a batch finish together (Sec. II, Eq. 1); the
 * pipeline has an SLO (Eq. 3); co-located pipelines share the GPU in space and
 * time through "inference streams" (Sec. III-C).  The paper leaves the execution
 * of a model to an inference engine; this library is that engine: letterbox,
 * convolution graphs, box decode, top-k, class-wise NMS, ROI compaction,
 * crop-resize and classifier tail as HIP kernels.
 *
 * Conventions
 *  - Plain C ABI.  Every call returns an octo_status; nothing throws or aborts.
 *  - "device" pointers are HIP device memory owned by the caller; "host" pointers
 *    are ordinary host memory.  The library allocates no device memory: the
 *    caller passes a workspace.  It does allocate pinned host memory for results.
 *  - Streams are passed as void* (hipStream_t).  Calls that take a stream only
 *    enqueue work on it.
 *  - NULL pointers, bad sizes or enum values give OCTO_EINVAL and change nothing.
 *  - One pipeline handle per host thread at a time; different handles may be used
 *    concurrently.
 */
#ifndef OCTO_H_
#define OCTO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OCTO_MAX_LEVELS 3
#define OCTO_MAX_ANCHORS 3
#define OCTO_MAX_EDGES 4
#define OCTO_MAX_CHILD_LABELS 2
#define OCTO_MAX_LAYER_INPUTS 4

typedef enum {
  OCTO_OK = 0,
  OCTO_EINVAL = -1,    /* bad argument */
  OCTO_ENOMEM = -2,    /* workspace too small / host allocation failed */
  OCTO_ECAP = -3,      /* a capacity was exceeded; results were clamped and flagged */
  OCTO_ESTATE = -4,    /* call not valid in the handle's current state */
  OCTO_EHIP = -5,      /* a HIP runtime call failed; see octo_last_error */
  OCTO_ENOTREADY = -6  /* non-blocking collect: nothing has finished yet */
} octo_status;

/* OCTO_F8 is 8-bit floating point in the OCP E4M3 format: 1 sign bit, 4 exponent bits (bias 7), 3 mantissa bits,
 * subnormals down to 2^-9, no infinities, 0x7F and 0xFF are NaN, largest finite value 448.  Only octo_op_conv and the
 * two conversion helpers below take it; models of a pipeline are stored in one of the other three. */
typedef enum { OCTO_F32 = 0, OCTO_F16 = 1, OCTO_BF16 = 2, OCTO_F8 = 3 } octo_dtype;
typedef enum { OCTO_CONV = 0, OCTO_MAXPOOL = 1, OCTO_UPSAMPLE2X = 2, OCTO_CONCAT = 3, OCTO_ADD = 4, OCTO_GAP = 5, OCTO_FC = 6 } octo_op;
typedef enum { OCTO_ACT_NONE = 0, OCTO_ACT_RELU = 1, OCTO_ACT_SILU = 2 } octo_act;
typedef enum { OCTO_RES_NONE = 0, OCTO_RES_BEFORE_ACT = 1, OCTO_RES_AFTER_ACT = 2 } octo_res_mode;
typedef enum { OCTO_DETECTOR = 0, OCTO_CLASSIFIER = 1 } octo_model_kind;

/* ---- records that live in device memory (also used by the stage-level calls) ---- */

/* One decoded detection candidate: corners in model-input pixels (not clamped). */
typedef struct { float x1, y1, x2, y2, score; int32_t cls; int32_t idx; int32_t pad_; } octo_cand;   /* 32 bytes */
/* One region of interest routed to a child model: source frame position in the batch,
 * rank in that frame's keep-list, class, corners in SOURCE pixels (clamped to the frame). */
typedef struct { int32_t frame, rank, cls, pad_; float x1, y1, x2, y2; } octo_roi;                   /* 32 bytes */
/* One final detection as returned by octo_collect: corners in source pixels. */
typedef struct { float x1, y1, x2, y2, score; int32_t cls; int32_t child_label[OCTO_MAX_CHILD_LABELS]; } octo_box;  /* 32 bytes */

/* ---- pipeline description (host memory; copied at create) ---- */

/* One layer of a model graph.  Tensor 0 is the model input (NHWC, in_c channels);
 * layer i produces tensor i+1.  conv: y = act(conv(x) + bias [+ res]) or act(conv(x) + bias) + res,
 * cross-correlation, zero padding.  fc is a 1x1 conv on a 1x1 map whose output stays fp32. */
typedef struct {
  int32_t op;                          /* octo_op */
  int32_t n_in;
  int32_t in[OCTO_MAX_LAYER_INPUTS];   /* tensor ids; conv with n_in == 2: in[1] is the residual */
  int32_t cout, kh, kw, stride, pad;
  int32_t act;                         /* octo_act */
  int32_t res_mode;                    /* octo_res_mode */
  const void* weight;                  /* host; [cout][kh][kw][cin] in the model's storage type (fp32 / IEEE half bits / bf16 bits) */
  const float* bias;                   /* host; fp32 [cout] */
} octo_layer;

/* One model (the paper's m).  batch_size is bz_m (Sec. II): the most items one launch processes. */
typedef struct {
  const char* name;
  int32_t dtype;                       /* octo_dtype: storage type of activations and weights; accumulation is fp32 */
  int32_t kind;                        /* octo_model_kind */
  int32_t in_h, in_w, in_c;            /* model input: letterbox target (root) or crop size (child) */
  const octo_layer* layers;
  int32_t n_layers;
  int32_t outputs[OCTO_MAX_LEVELS];    /* detector: head tensors, largest grid first; classifier: outputs[0] = fp32 logits */
  int32_t n_outputs;
  /* detector post-processing */
  int32_t n_classes, n_anchors;
  int32_t stride[OCTO_MAX_LEVELS];
  float anchors[OCTO_MAX_LEVELS][OCTO_MAX_ANCHORS][2];   /* (w, h) in model-input pixels */
  float score_thr, iou_thr;            /* keep iff score > score_thr; suppress iff inter > iou_thr * union (same class) */
  int32_t topk, max_det;               /* threshold -> top-k -> NMS -> cut to max_det */
  /* pre-processing of this model's input */
  float norm_scale[3], norm_bias[3];   /* out = pixel * scale + bias per channel */
  int32_t pad_value;                   /* letterbox padding colour (0..255) */
  int32_t batch_size;
} octo_model_desc;

/* DAG edge (Sec. II: models form a DAG): detections of `parent` whose class bit is set go to `child`. */
typedef struct { int32_t parent, child; uint64_t class_mask[2]; } octo_edge;

typedef struct {
  const octo_model_desc* models; int32_t n_models;    /* models[0] is the root detector; a later model without an incoming
                                                         edge is detached (runs only through octo_debug_run_model) */
  const octo_edge* edges; int32_t n_edges;
  float slo_ms;                                       /* SLO_p (Eq. 3) */
  int32_t src_h, src_w;                               /* camera frame size; frames are uint8 HWC RGB */
  int32_t max_frames;                                 /* capacity of one detector batch (>= models[0].batch_size) */
  int32_t max_rois_per_frame;                         /* per-edge ROI capacity = max_frames * max_rois_per_frame */
  int32_t max_queue;                                  /* submitted-but-not-run frames; 0 = 4 * max_frames */
  int32_t keep_all_tensors;                           /* != 0: every tensor gets its own memory, so octo_debug_get_tensor can
                                                         read any of them after a run (otherwise only model outputs are safe).
                                                         1: and every layer runs on its own, so every tensor is written;
                                                         2: layers are fused as in normal operation (a first layer followed by
                                                         a 3x3 / stride-2 max-pool writes only the pooled tensor; the tensor
                                                         in between then holds nothing; two consecutive 1x1 convolutions of
                                                         one input with one activation run as one launch) */
} octo_pipeline_desc;

typedef struct octo_pipeline octo_pipeline;

/* Result of one frame.  latency_ms = completion - arrival on the clock of octo_now_ms; all frames of a batch
 * complete together (Sec. II).  slo_met = latency_ms <= slo_ms (effective throughput counts these, Sec. II). */
typedef struct { int64_t frame_id; int32_t n_boxes; float latency_ms; int32_t slo_met; int32_t flags; int32_t box_offset; int32_t pad_; } octo_frame_result;
#define OCTO_FLAG_ROI_OVERFLOW 1
#define OCTO_FLAG_CAND_OVERFLOW 2

/* ---- the serving calls ---- */

/* Device bytes octo_pipeline_create needs for this description (activations of every model at its capacity,
 * packed weights, post-processing tables).  Host only. */
octo_status octo_pipeline_workspace_size(const octo_pipeline_desc* desc, size_t* device_bytes);

/* Build a pipeline.  `device_workspace` (256-byte aligned, `bytes` long, caller-owned, must outlive the handle)
 * receives packed weights (copied synchronously) and all intermediate tensors.  OCTO_ENOMEM if too small. */
octo_status octo_pipeline_create(const octo_pipeline_desc* desc, void* device_workspace, size_t bytes, octo_pipeline** out);
octo_status octo_pipeline_destroy(octo_pipeline* p);

/* Queue n frames.  d_frames[i] is a device pointer to uint8 [src_h][pitch_bytes[i]] with 3*src_w valid bytes per row;
 * the arrays themselves are host memory.  Frame memory must stay valid until the frame has been collected.
 * arrival_ms uses the clock of octo_now_ms.  OCTO_ECAP (nothing queued) if the queue would overflow. */
octo_status octo_submit_frames(octo_pipeline* p, const void* const* d_frames, const size_t* pitch_bytes,
                               const double* arrival_ms, const int64_t* frame_ids, int32_t n);

/* Form one batch of up to bz (models[0].batch_size, or the value set by octo_set_batch_size) queued frames in
 * arrival order and enqueue the whole cascade for it on `hip_stream`; no host-device synchronisation.
 * *n_frames_launched = 0 and OCTO_OK if the queue is empty; OCTO_ESTATE if too many batches (7) are uncollected. */
octo_status octo_run(octo_pipeline* p, void* hip_stream, int32_t* n_frames_launched);

/* Fetch finished batches, oldest first.  frames[0..*n_frames) and boxes[0..*n_boxes) are host arrays; a frame's
 * boxes are boxes[box_offset .. box_offset + n_boxes) in keep-list (score) order.  blocking != 0 waits for the
 * oldest batch; otherwise OCTO_ENOTREADY if none has finished.  A batch is only returned if it fits entirely. */
octo_status octo_collect(octo_pipeline* p, octo_frame_result* frames, int32_t frame_cap, octo_box* boxes, int32_t box_cap,
                         int32_t* n_frames, int32_t* n_boxes, int32_t blocking);

/* The batch size of the root model: the most frames one batch takes from the queue (1 <= bz <= max_frames).  Downstream
 * models have no launch batch size: a child runs once per batch on however many ROIs its parent emitted, the count
 * staying on the device; a scheduler's batch size for a child (Algorithm 1) only sizes its time slot.  model > 0 is
 * therefore refused with OCTO_EINVAL. */
octo_status octo_set_batch_size(octo_pipeline* p, int32_t model, int32_t bz);
/* Every model has a batch size of its own (Sec. III-B, Algorithm 1): with frames_per_execution = b > 0 the detector's
 * layers and post-processing run on b frames at a time, ceil(n / b) executions per batch of n frames, while the
 * downstream models still run once on the ROIs of the whole batch - a detector at batch size b feeding children that
 * batch the objects of several of its executions.  0 (the default): one execution for the whole batch.  Results are
 * identical either way.  Layer tensors read back with octo_debug_get_tensor, and the per-layer times, are those of
 * the last execution.  0 <= b <= max_frames. */
octo_status octo_set_detector_batch(octo_pipeline* p, int32_t frames_per_execution);
const char* octo_last_error(const octo_pipeline* p);    /* library-owned text, valid until the next call on p (NULL p: last create error) */
double octo_now_ms(void);                               /* monotonic host clock used for arrival / completion times */

/* Spatial sharing (Sec. III-C: a stream's width is its share of compute): create / destroy a HIP stream
 * restricted to the compute units whose bit is set (cu_mask: n_words 32-bit words), default priority. */
octo_status octo_stream_create_masked(const uint32_t* cu_mask, int32_t n_words, void** hip_stream);
/* The same for the contiguous unit range [first_cu, first_cu + n_cu), both multiples of 8: mask bit i selects unit
 * i / 8 of die i % 8 on this GPU, so such a range is an equal slice of every die and two disjoint ranges share no
 * compute unit.  OCTO_EINVAL for a mask or range that leaves a die without units (the runtime refuses those). */
octo_status octo_stream_create_range(int32_t first_cu, int32_t n_cu, void** hip_stream);
octo_status octo_stream_destroy(void* hip_stream);
octo_status octo_device_cu_count(int32_t* n_cu);

/* ---- scheduling (host only; Algorithm 1 batch-size part and Algorithm 2 of the paper) ---- */

typedef struct {
  int32_t parent;                 /* index of the upstream model in the pipeline, -1 for the root */
  int32_t n_profile;              /* profiled batch sizes (ascending powers of two starting at 1) */
  int32_t profile_bz[8];
  float profile_ms[8];            /* L_{m|bz}: batch latency in ms */
  float rate;                     /* requests per second reaching the model */
  float burstiness;               /* coefficient of variation of inter-arrival times (Sec. III-B) */
  float util;                     /* U_m: share of GPU compute (portion width), 0..1 */
  float weight_mem, inter_mem;    /* W_m, I_m (any one unit) */
  int32_t bz;                     /* in/out: chosen batch size */
} octo_sched_model;

typedef struct { octo_sched_model* models; int32_t n_models; float slo_ms; } octo_sched_pipeline;
typedef struct { int32_t pipeline, model, stream; float start_ms, end_ms, duty_cycle_ms; } octo_placement;  /* stream -1: not placed */

/* Algorithm 1, batch-size search with device and GPU fixed and one instance per model: start at bz = 1, visit
 * models from the burstiest down, double, drop if the estimated latency exceeds SLO/2, adopt if the estimated
 * throughput improves, repeat until a sweep adopts nothing.  Writes models[i].bz. */
octo_status octo_cwd_search(octo_sched_pipeline* p);
/* Algorithm 2: per model (pipelines in order, models in order) the tightest free portion that contains the
 * model's window, keeps memory and utilisation within the GPU and whose stream's duty cycle is not longer
 * than SLO/2.  out has sum(n_models) entries. */
octo_status octo_coral_schedule(octo_sched_pipeline* ps, int32_t n_pipelines, double gpu_mem, double util_max,
                                int32_t n_streams, octo_placement* out);
float octo_est_latency_ms(const octo_sched_pipeline* p);
float octo_est_throughput(const octo_sched_pipeline* p);

/* ---- run-time rules of the serving loop (host only) ----
 * The paper names them in prose; each comment states the reading this library takes. */

/* Burstiness of a request stream (Sec. III-B: the coefficient of variation of inter-request arrival times): population
 * standard deviation / mean of the gaps between the n arrival times taken in ascending order; 0 for fewer than three
 * arrivals or a zero mean gap. */
octo_status octo_burstiness(const double* times, int32_t n, double* cv);
/* Back-to-back batches a model's portion must hold with one instance per model (Sec. III-C: a portion is as long as the
 * model's execution): ceil(rate x duty cycle / bz), at least 1. */
octo_status octo_batches_per_cycle(double rate_per_s, double duty_ms, int32_t bz, int32_t* k);
/* Portion width (share of the GPU's compute, Sec. III-C) -> compute units: rounded up to whole multiples of `grain`
 * (8 on this GPU: one unit per die), at least one grain, at most total_cus. */
octo_status octo_width_to_cus(double util, int32_t total_cus, int32_t grain, int32_t* n_cu);
/* Width of a model from its batch latency on streams of n widths (compute units).  by_cost != 0: the narrowest width
 * whose cost width x latency is within tol of the cheapest (a model that does not speed up on more units should not
 * hold them); by_cost == 0: the narrowest width whose latency is within tol of the widest width's. */
octo_status octo_choose_width(const int32_t* widths, const double* latency_ms, int32_t n, int32_t by_cost, double tol, int32_t* width);
/* Load-aware widths around Algorithm 1 (Sec. III-C takes a model's measured utilisation as its width and does not say
 * what happens when a pipeline's work does not fit its duty cycle at those widths).  models[i].width is the width the
 * model's own profile chose (octo_choose_width; one of widths[]), profile_ms[j][k] its batch latency at widths[j] and
 * batch size profile_bz[k].  For every profiled width taken as a floor, in ascending order: each model runs at
 * max(floor, its own width); octo_cwd_search picks the batch sizes with the latencies of those widths (fixed_bz != NULL:
 * these are taken instead); a model needs octo_batches_per_cycle batches per cycle; the floor is accepted if the
 * pipeline's work per duty cycle, sum k x L(bz), is at most cycle_share x duty_ms, and the widest floor whatever its work.
 * out[i]: the model as Algorithm 2 takes it - util = width / total_cus, bz, and the batch latency at bz multiplied by
 * k (its portion holds k back-to-back batches); the two estimates are taken before that multiplication. */
#define OCTO_MAX_WIDTHS 4
typedef struct {
  int32_t parent;
  float rate, burstiness, weight_mem, inter_mem;
  int32_t width;
  int32_t n_profile; int32_t profile_bz[8];
  float profile_ms[OCTO_MAX_WIDTHS][8];
} octo_plan_model;
octo_status octo_plan_pipeline(const octo_plan_model* models, int32_t n_models, float slo_ms, double duty_ms, double cycle_share,
                               const int32_t* widths, int32_t n_widths, int32_t total_cus, const int32_t* fixed_bz,
                               octo_sched_model* out, int32_t* batches_per_cycle, float* est_latency_ms, float* est_throughput);
/* Cross-device placement of one pipeline (Algorithm 1, function ToEdge, Sec. III-B) for two devices: the server and the
 * edge device at the data source, joined by a link of bandwidth_bytes_per_s.  In: every model on the server with the
 * batch size octo_cwd_search chose (bz, one of profile_bz).  Depth first from the root: a model moves to the edge if a
 * configuration for it exists there, its downstream models are then tried (least bursty first), and on the way back it
 * returns to the server if alpha x (bytes/s entering it) < (bytes/s leaving it) while none of its downstream models is
 * on the edge (Insights 2 and 3).  Out: on_edge and bz per model, and the two estimates of the result.
 * Readings of what the paper leaves open: the estimates are octo_est_latency_ms / octo_est_throughput plus Eq. (1)'s
 * network term - a model fed from the other device (the root is fed by the data source, at the edge) pays
 * in_bytes / bandwidth per request; "a configuration on the edge" changes only that model's device and batch size and
 * takes, among the profiled batch sizes that keep the latency estimate within slo_ms / 2 and the edge device within its
 * compute (sum over edge models of rate x L(bz) / bz <= one second per second), the one with the largest throughput
 * estimate, the smallest on ties; bytes/s leaving a model = sum over its downstream models of rate x in_bytes, for a
 * leaf rate x result_bytes. */
typedef struct {
  int32_t parent;                 /* -1 for the root (model 0); parents precede children */
  float rate, burstiness;
  int32_t n_profile; int32_t profile_bz[8];      /* ascending */
  float server_ms[8], edge_ms[8]; /* batch latency on either device */
  double in_bytes;                /* size of one request entering the model */
  double result_bytes;            /* size of one result leaving the pipeline at this model (leaves) */
  int32_t bz;                     /* in/out */
  int32_t on_edge;                /* out */
} octo_place_model;
octo_status octo_to_edge(octo_place_model* models, int32_t n_models, float slo_ms, double bandwidth_bytes_per_s, double alpha,
                         float* est_latency_ms, float* est_throughput);
/* Lazy dropping (Sec. IV-A): how many requests at the head of an arrival-ordered queue are already older than the
 * objective when a batch is formed (now - arrival > slo; exactly the objective old is still served; counting stops
 * at the first request that is not late). */
octo_status octo_late_prefix(const double* arrival_ms, int32_t n, double now_ms, double slo_ms, int32_t* n_late);
/* Horizontal scaling between two runs of the scheduler (Sec. III-D).  One object per pipeline; once per duty cycle
 * octo_scaler_observe is told how many requests arrived and how many are queued, with n_active instances running, each
 * serving `capacity` requests per cycle.  Over the last `window` cycles: *decision = +1 if n_active < max_instances and
 * (mean arrivals > up x capacity x n_active, or the queue never fell to capacity x n_active or below); else -1 if
 * n_active > 1, mean arrivals < down x capacity x (n_active - 1) and the current queue fits capacity x (n_active - 1);
 * else 0.  A non-zero decision empties the window; before the window is full the decision is 0.  down < up. */
typedef struct octo_scaler octo_scaler;
octo_status octo_scaler_create(double capacity, int32_t window, double up, double down, int32_t max_instances, octo_scaler** out);
octo_status octo_scaler_observe(octo_scaler* s, int64_t arrived, int64_t backlog, int32_t n_active, int32_t* decision);
octo_status octo_scaler_destroy(octo_scaler* s);

/* Temporal sharing: run only model `model` of the pipeline on `hip_stream` (used by a slot executor that places
 * each model's portion itself).  Model 0 forms the batch as octo_run does and stops after ROI compaction;
 * a child model consumes the ROIs of the most recent model-0 run; after the last child the batch becomes
 * collectable.  octo_run is the same sequence on one stream. */
octo_status octo_run_model(octo_pipeline* p, int32_t model, void* hip_stream, int32_t* n_items_launched);

/* ---- slot executor (Sec. III-C "Inference Stream", Sec. III-D, Sec. IV-A) ----
 * Serves several pipelines on one GPU from a schedule: every duty cycle, at the start of an instance's portion
 * (slot_ms), its detector is launched on what is queued for it - at most bz frames per batch and batches_per_cycle + 1
 * batches per slot - and its downstream models follow on the streams of their own portions (octo_run_model).  Requests
 * come from cameras: arrival times in seconds from the start of serving and a pool of device frames each camera cycles
 * through.  All descriptor arrays are host memory and are copied at create; frames, head pools and head buffers are
 * device memory the caller keeps alive until destroy.  One executor per host thread. */
typedef struct {
  int32_t bz;                     /* frames per detector batch (Algorithm 1's choice for the root model) */
  int32_t batches_per_cycle;      /* octo_batches_per_cycle of the root model */
  float slo_ms;
  /* planted heads (parity and benchmark mode; n_levels = 0: none): head_pool[l] is [pool items][head_item_bytes[l]]; before
   * a batch runs, the items of the batch's frames are copied into the instance's head_buffers, which decode reads */
  const void* const* head_pool;
  const size_t* head_item_bytes;
  int32_t n_levels;
  /* scaler of the queue's stand-by instance (0: window 5, up 1.0, down 0.75); capacity = (batches_per_cycle + 1) * bz */
  int32_t scaler_window;
  float scaler_up, scaler_down;
} octo_exec_queue;

typedef struct {
  octo_pipeline* pipe;
  int32_t queue;                  /* the request queue it serves */
  int32_t standby;                /* != 0: a stand-by copy, switched on and off by the queue's scaler (slotted mode only) */
  void* const* streams;           /* [n_models]: HIP stream of each model's portion */
  int32_t n_models;
  float slot_ms;                  /* start of its first model's portion inside the duty cycle */
  void* const* head_buffers;      /* [n_levels] device buffers installed with octo_debug_set_head, or NULL */
  int32_t max_frames, max_batch, max_det;   /* of its pipeline: frame capacity, largest detector batch, boxes kept per frame */
} octo_exec_instance;

typedef struct {
  int32_t queue;
  const double* arrivals_s; int32_t n_arrivals;       /* ascending */
  const void* const* d_frames; const size_t* pitch_bytes; int32_t n_frames;   /* request k shows frame k % n_frames */
  int32_t pool_offset;            /* index of its first frame in the queue's head pool */
} octo_exec_camera;

typedef struct {
  const octo_exec_queue* queues; int32_t n_queues;
  const octo_exec_instance* instances; int32_t n_instances;      /* scheduled instances first (one per queue), then stand-by copies */
  const octo_exec_camera* cameras; int32_t n_cameras;
  float duty_ms;
  int32_t slotted;                /* 0: no portions - every instance launches as soon as something is queued */
  int32_t drop_late;              /* lazy dropping (octo_late_prefix) when a batch is formed */
  int32_t keep_results;           /* keep every served frame's boxes for octo_executor_results */
  /* for placing stand-by copies (NULL / 0 without them): Algorithm 2's inputs for the scheduled pipelines, one per queue,
   * and the streams its placements refer to (schedule stream index -> handle and compute-unit range) */
  const octo_sched_pipeline* sched; double gpu_mem; int32_t n_streams;
  const int32_t* stream_index; void* const* stream_handle; const int32_t* stream_first_cu; const int32_t* stream_n_cu; int32_t n_sched_streams;
  int32_t masked;                 /* != 0: a newly placed copy's stream is restricted to its compute-unit range; 0: plain_stream is used */
  void* plain_stream;
} octo_exec_desc;

typedef struct {
  int64_t submitted, served, slo_met, boxes, dropped;   /* dropped: late requests removed at batch formation */
  float latency_ms_p50, latency_ms_p99, latency_ms_max;
} octo_exec_stats;
typedef struct { float t_s; int32_t queue; int32_t change; } octo_scale_event;   /* +1 copy switched on, -1 off, 0 no room for it */

typedef struct octo_executor octo_executor;
/* Also runs one frame through every instance (warm-up).  OCTO_EINVAL for an inconsistent description. */
octo_status octo_executor_create(const octo_exec_desc* desc, octo_executor** out);
/* Serve the arrivals earlier than duration_s, then wait up to drain_s for the queues to empty; blocking.
 * *wall_s = time from the first slot to the end of the loop.  Statistics add up over calls. */
octo_status octo_executor_serve(octo_executor* ex, double duration_s, double drain_s, double* wall_s);
octo_status octo_executor_stats(const octo_executor* ex, int32_t queue, octo_exec_stats* out);
octo_status octo_executor_scale_events(const octo_executor* ex, octo_scale_event* out, int32_t cap, int32_t* n);
/* Streams in use: those of the schedule plus the ones created for placed copies (schedule stream index, compute-unit range). */
octo_status octo_executor_streams(const octo_executor* ex, int32_t* stream_index, int32_t* first_cu, int32_t* n_cu, int32_t cap, int32_t* n);
/* keep_results: every served frame of a queue - request id (arrival order), index in the head pool / camera pools, and its
 * boxes boxes[box_offset .. box_offset + n_boxes).  OCTO_ECAP (with the needed sizes in *n_frames, *n_boxes_total) if too small. */
octo_status octo_executor_results(const octo_executor* ex, int32_t queue, int64_t* frame_ids, int32_t* pool_index, int32_t* box_offset,
                                  int32_t* n_boxes, int32_t frame_cap, octo_box* boxes, int32_t box_cap, int32_t* n_frames, int32_t* n_boxes_total);
const char* octo_executor_last_error(const octo_executor* ex);
octo_status octo_executor_destroy(octo_executor* ex);

/* ---- profiling and parity hooks ---- */

/* Time every layer of a model: each layer is launched `iters` times back to back between two HIP events on
 * `hip_stream` for `n` items; ms[i] = mean duration of layer i, flops[i] / bytes[i] its dense FLOPs and the
 * element bytes of its external tensors (activations of n items plus weights once).  Synchronises the stream. */
octo_status octo_profile_layers(octo_pipeline* p, int32_t model, int32_t n, int32_t iters, void* hip_stream,
                                float* ms, double* flops, double* bytes, int32_t cap);
/* Per-layer GPU time inside the serving path: after octo_set_layer_timing(p, 1) every run records a HIP event
 * between the layers of each model (on the stream the layers run on); octo_get_layer_info then returns, for the most
 * recently collected batch, ms[i] = run time of layer i (convolution and fully connected layers: the kernel's own
 * duration, from events attached to its dispatch; other layers: end of layer i-1 to end of layer i on the stream,
 * which includes the launch gap), kernel_id[i] = which kernel ran it (general convolution: decimal digits
 * 1 BBB PPP K M V = channel tile, pixel tile, 16-byte vectors per K step, workgroups per CU, V = vectorised gather
 * + 2 if operands go straight to LDS; 17 0P BBB TTT: wide 3x3 kernel, channel tile BBB, tile width TTT, P = 1 for 512-pixel tiles (else 256);
 * 18 00 BBB 0 SS: 3x3 kernel with the input patch in LDS, channel tile BBB and
 * channel slice SS; 19 0F BBB KK P: first-layer kernel, channel tile, kernel height, kernel width in pixel pairs,
 * F = 1 when it also computes the 3x3 / stride-2 max-pool that follows (that layer then reports kernel 0 and 0 ms);
 * 1 max-pool, 2 upsample, 3 channel copy, 4 add, 5 global average pool, 0 none), per ITEM dense FLOPs and activation
 * bytes (input, output and residual elements), and per LAUNCH weight and bias bytes.  When two 1x1 convolutions of
 * the same input run as one launch, the first reports the kernel, the time and the work of both (the shared input
 * counted once) and the second kernel 0 and no work. */
octo_status octo_set_layer_timing(octo_pipeline* p, int32_t enable);
octo_status octo_get_layer_info(octo_pipeline* p, int32_t model, float* ms, int32_t* kernel_id, double* flops, double* bytes,
                                double* weight_bytes, int32_t cap, int32_t* n);
/* Per-stage GPU time of the most recently collected batch, ms: letterbox, detector layers, decode, top-k, NMS,
 * compaction, then per edge (crop, child layers, child post-processing).  Only measured after
 * octo_set_stage_timing(p, 1), which adds event records between stages. */
octo_status octo_set_stage_timing(octo_pipeline* p, int32_t enable);
octo_status octo_get_stage_ms(octo_pipeline* p, float* ms, int32_t cap, int32_t* n);

/* Microbenchmarks of the GPU itself, for "fraction of what this machine sustains" beside the datasheet fractions.
 * octo_probe_copy: a plain 16-byte-per-lane copy of `bytes` from d_src to d_dst (device, 16-byte aligned), `reps`
 * timed passes after a warm-up; *gb_per_s = (bytes read + bytes written) / median time.
 * octo_probe_mfma: a register-only loop of the 32x32x16 matrix instruction of `dtype` (OCTO_F16 / OCTO_BF16; for
 * OCTO_F8 the 32x32x64 instruction on E4M3 operands) with
 * random operand values, 16 independent accumulators per wavefront, one workgroup of four wavefronts per compute
 * unit, `iters` x 16 instructions per wavefront; d_scratch (device, at least CUs x 1 KiB) receives checksums;
 * *tflops = dense FLOP / median time.  Both synchronise `hip_stream`. */
octo_status octo_probe_copy(const void* d_src, void* d_dst, size_t bytes, int32_t reps, void* hip_stream, double* gb_per_s);
octo_status octo_probe_mfma(int32_t dtype, float* d_scratch, size_t scratch_bytes, int32_t iters, int32_t reps, void* hip_stream, double* tflops);

/* Copy items [first_item, first_item + n_items) of a tensor of the last run to host as dense NHWC in the tensor's
 * type (fp32 for fc outputs).  tensor_id as in octo_layer.  Synchronises the device. */
octo_status octo_debug_get_tensor(octo_pipeline* p, int32_t model, int32_t tensor_id, int32_t first_item, int32_t n_items,
                                  void* host_dst, size_t bytes);
octo_status octo_debug_tensor_shape(octo_pipeline* p, int32_t model, int32_t tensor_id, int32_t* h, int32_t* w, int32_t* c);
/* Replace (d_head != NULL) or restore (NULL) the head tensor of `level` that decode reads: dense
 * [items][G][G][A*(5+C)] in the model's type, device memory owned by the caller. */
octo_status octo_debug_set_head(octo_pipeline* p, int32_t model, int32_t level, const void* d_head);
/* Run one model on a caller-provided dense input [n][in_h][in_w][in_c] (device, model's type). */
octo_status octo_debug_run_model(octo_pipeline* p, int32_t model, const void* d_input, int32_t n, void* hip_stream);
/* Copy post-processing tables of the last batch to host (synchronises): per item candidate count, top-k list,
 * keep-list; per edge ROI table. */
octo_status octo_debug_get_detections(octo_pipeline* p, int32_t model, int32_t item, int32_t* cand_count,
                                      octo_cand* top, int32_t top_cap, int32_t* n_top, int32_t* keep, int32_t keep_cap, int32_t* n_keep);
octo_status octo_debug_get_rois(octo_pipeline* p, int32_t edge, octo_roi* rois, int32_t cap, int32_t* n_rois);
octo_status octo_debug_get_labels(octo_pipeline* p, int32_t edge, int32_t* labels, int32_t cap, int32_t* n);

/* ---- stage-level calls: the same kernels the pipeline launches, on caller-owned device buffers ---- */

/* Where the letterbox puts a src_h x src_w frame inside a dst_h x dst_w input (host only, no GPU): the resized
 * frame is *nw x *nh pixels (r = min(dst_w / src_w, dst_h / src_h), sizes rounded half up) with its top-left corner
 * at (*left, *top), centred with the odd pixel going right / down.  Boxes are mapped back with exactly these values. */
octo_status octo_letterbox_geometry(int32_t src_h, int32_t src_w, int32_t dst_h, int32_t dst_w,
                                    int32_t* nw, int32_t* nh, int32_t* left, int32_t* top);

/* Letterbox + normalise: aspect-preserving bilinear resize (half-pixel centres, no antialias) of n uint8 HWC
 * frames into dst [n][dst_h][dst_w][3] of `dtype`, centred, padded with pad_value, out = px*scale + bias.
 * d_frame_ptrs / d_pitches: device arrays of n frame pointers / row pitches. */
octo_status octo_op_letterbox(const void* d_frame_ptrs, const void* d_pitches, int32_t n, int32_t src_h, int32_t src_w,
                              void* d_dst, int32_t dst_h, int32_t dst_w, int32_t dtype, const float* scale3, const float* bias3,
                              int32_t pad_value, void* hip_stream);
/* Crop-resize: for ROI j < min(*d_n_rois, cap) bilinear stretch of its source box from frame rois[j].frame
 * (clamped to 0..n_frames-1) into dst [cap][out_h][out_w][3]. */
octo_status octo_op_crop_resize(const void* d_frame_ptrs, const void* d_pitches, int32_t n_frames, int32_t src_h, int32_t src_w,
                                const octo_roi* d_rois, const int32_t* d_n_rois, int32_t cap,
                                void* d_dst, int32_t out_h, int32_t out_w, int32_t dtype, const float* scale3, const float* bias3,
                                void* hip_stream);
/* One convolution layer, batched over n items (the model execution whose batch latency L_m(bz) Eq. (1) is about; the
 * pipeline runs its layers through the same kernels):
 *   y[i,p,q,k] = act(bias[k] + sum_{r,s,c} x[i, p*stride + r - pad, q*stride + s - pad, c] * w[k,r,s,c]  (+ residual))
 * on NHWC device tensors of `dtype`, accumulated in fp32.  x: [n][h][w] pixels x_ld elements apart (x_ld >= cin),
 * y: [n][ho][wo] pixels y_ld apart with ho = (h + 2 pad - kh) / stride + 1, residual (or NULL) shaped like y with pitch
 * res_ld, added before or after the activation (octo_res_mode).  out_f32 != 0 writes y as fp32 instead of `dtype`.
 * d_w: the weights in the packed layout octo_op_conv_pack makes (device copy of it, octo_op_conv_packed_bytes long);
 * d_bias: device, octo_op_conv_padded_cout(cout) floats, zero beyond cout.  The library keeps no pointer after the
 * launch.  *kernel_id (may be NULL) receives the id of the kernel chosen (see octo_get_layer_info).
 * OCTO_F8 (not from the paper: a reduced-precision variant of the same kernel on the 8-bit matrix instructions):
 * x, w, residual and y hold E4M3 codes; real value = code value times a scale the caller chose.
 *   y_real = act(acc * d_scale[k] + bias[k]  (+ res_code_value * res_scale)),   y_code = E4M3(y_real * y_inv_scale)
 * with d_scale (device, padded like the bias) = weight scale of channel k times the scale of x; the conversion rounds
 * to nearest even and saturates at +-448 (what a NaN result is stored as is not specified).  cin and x_ld must be
 * multiples of 16 (OCTO_EINVAL otherwise); y_ld and res_ld may be anything, but pitches that are no multiple of 16
 * (y) or 4 (residual) take a slower element-wise path.  For the other types d_scale, res_scale and y_inv_scale are
 * ignored, and any cin / pitch is accepted (channel counts or pitches that are no multiple of 8, 4 for fp32, are
 * gathered element by element).
 * All types: d_x, d_w, d_y and d_res must be 16-byte aligned; res_mode and d_res must agree (both or neither).
 * Errors: OCTO_EINVAL for null / non-positive / misaligned arguments and for shapes beyond the kernel's 32-bit
 * offsets (two images plus 1024 strided pixels of x must stay below 2 GiB; n*ho*wo below 2^31; K padded below 65536);
 * nothing is launched then.  The call only enqueues on hip_stream. */
typedef struct octo_conv_op {
  int32_t dtype;
  int32_t n, h, w, cin, x_ld;
  int32_t cout, kh, kw, stride, pad;
  int32_t act, res_mode, out_f32;
  int32_t y_ld, res_ld;
  const void* d_x;
  const void* d_w;
  const float* d_bias;
  const float* d_scale;
  const void* d_res;
  void* d_y;
  float res_scale, y_inv_scale;
} octo_conv_op;
octo_status octo_op_conv(const octo_conv_op* op, void* hip_stream, int32_t* kernel_id);
/* Packed weight layout (host only, no GPU).  w: [cout][kh][kw][cin] in `dtype` (host).  packed: host buffer of
 * octo_op_conv_packed_bytes(...) bytes, fully written (rows padded to whole K steps and the row count to
 * octo_op_conv_padded_cout(cout), zero filled).  Copy it to the device as it is. */
size_t octo_op_conv_packed_bytes(int32_t dtype, int32_t cout, int32_t kh, int32_t kw, int32_t cin);
int32_t octo_op_conv_padded_cout(int32_t cout);
octo_status octo_op_conv_pack(int32_t dtype, const void* w, int32_t cout, int32_t kh, int32_t kw, int32_t cin, void* packed);
/* E4M3 conversion on the host (no GPU): dst[i] = E4M3(src[i] * inv_scale), round to nearest even, saturating at
 * +-448, NaN -> 0x7F; and back: dst[i] = value(src[i]) * scale (NaN codes give NaN). */
octo_status octo_quantize_e4m3(const float* src, size_t n, float inv_scale, uint8_t* dst);
octo_status octo_dequantize_e4m3(const uint8_t* src, size_t n, float scale, float* dst);
/* Decode + threshold of n items: d_heads[l] dense [n][G_l][G_l][A*(5+C)].  Appends candidates with
 * score > thr to d_cand[item*cap ...] (order unspecified), d_count[item] = number found (may exceed cap:
 * then only cap were stored).  Geometry and thresholds are read from `model`. */
octo_status octo_op_decode(const octo_model_desc* model, const void* const* d_heads, int32_t n,
                           octo_cand* d_cand, int32_t* d_count, int32_t cap, void* hip_stream);
/* Top-k of each item's list by (score descending, idx ascending): d_out[item*k_cap ...] sorted, d_out_count[item]
 * = min(count, k).  k <= k_cap. */
octo_status octo_op_topk(const octo_cand* d_in, const int32_t* d_in_count, int32_t in_cap, int32_t n, int32_t k,
                         octo_cand* d_out, int32_t* d_out_count, int32_t k_cap, void* hip_stream);
/* Greedy class-wise NMS over sorted lists; d_keep[item*max_det ...] = kept positions ascending, cut to max_det.
 * d_mask_scratch: octo_op_nms_scratch_bytes(n, k_cap) bytes.  k_cap must be a multiple of 64, at most 4096. */
octo_status octo_op_nms(const octo_cand* d_top, const int32_t* d_top_count, int32_t k_cap, int32_t n, float iou_thr, int32_t max_det,
                        void* d_mask_scratch, int32_t* d_keep, int32_t* d_n_keep, void* hip_stream);
size_t octo_op_nms_scratch_bytes(int32_t n, int32_t k_cap);
/* octo_op_nms for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): same arguments, results and kernels, but the suppression mask lives in a static
 * device array inside the library (OCTO_NMS_STATIC_BYTES per GPU, held until the process ends) and the call itself
 * allocates nothing.  OCTO_ECAP, with nothing launched, if octo_op_nms_scratch_bytes(n, k_cap) exceeds
 * OCTO_NMS_STATIC_BYTES (e.g. 64 items at k_cap 1024 fit exactly).  All calls on one GPU share the array: calls
 * that overlap on one GPU (different streams, or different threads) race; calls on one stream are ordered.  The
 * array keeps the previous call's contents; none of them is read (each call writes every mask word it reads). */
#define OCTO_NMS_STATIC_BYTES (8u << 20)
octo_status octo_op_nms_static(const octo_cand* d_top, const int32_t* d_top_count, int32_t k_cap, int32_t n, float iou_thr, int32_t max_det,
                               int32_t* d_keep, int32_t* d_n_keep, void* hip_stream);
/* ROI compaction for one edge: kept boxes with class bit set, in (item, rank) order, converted to source pixels
 * (letterbox undone for a src_h x src_w frame letterboxed into in_h x in_w) and clamped.
 * d_n_rois[0] = count (clamped to cap); d_roi_of [n][max_det] = ROI id of each kept box or -1; d_item_counts [n] is
 * scratch; d_boxes [n][max_det] (may be NULL) receives every kept box in source pixels; d_flags [n] may be NULL. */
octo_status octo_op_compact(const octo_cand* d_top, int32_t k_cap, const int32_t* d_keep, const int32_t* d_n_keep, int32_t max_det,
                            int32_t n, int32_t src_h, int32_t src_w, int32_t in_h, int32_t in_w, const uint64_t* class_mask2,
                            octo_roi* d_rois, int32_t* d_n_rois, int32_t cap, int32_t* d_roi_of, int32_t* d_item_counts, octo_box* d_boxes,
                            int32_t* d_flags, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* OCTO_H_ */
