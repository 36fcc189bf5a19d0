/*
 * vpe.h -- C ABI of the MI355X-native Visual Perception Engine hot path.
 *
 * The paper's engine (Sec. "System architecture") is a foundation module that runs a
 * vision backbone continuously and writes its features into a "middle buffer", plus any
 * number of head modules that read those features by reference, each at its own
 * adjustable rate, with all buffers preallocated at start-up.  This library is that
 * data path on one AMD MI355X (gfx950) in one process: the encoder writes each frame's
 * features ONCE into a slot of a preallocated device ring; heads read the slot IN PLACE
 * (no copies) on their own HIP streams; ordering is by HIP events.
 *
 * Every compute step behind these calls is a hand-written HIP kernel.  The library never
 * touches host copies of activations and never allocates device memory after vpe_create.
 *
 * Conventions
 *   - return value: 0 = VPE_OK, 1 = VPE_SKIPPED (head not due on that frame; not an
 *     error), 2 = VPE_BUSY (vpe_run_head_latest only: the head's previous run has not finished; not an
 *     error), negative = error (see vpe_status).  vpe_last_error() gives a message.
 *   - "device" pointers are HIP device addresses on the current device; "host" pointers
 *     are ordinary process memory.
 *   - streams are hipStream_t passed as void*; NULL selects the engine's own stream for
  *     that call (one stream per encoder lane, one stream per head, all at default priority).
 *   - vpe_encode and vpe_run_head only enqueue work; vpe_sync blocks until it is done.
 *   - an engine may be driven from one host thread at a time.
 *
 * Throughput.  With the defaults (encoder_lanes = 1) frames pass through the encoder one after another and a
 * ViT-S pass leaves most of the 256 compute units idle (about 1000 frames/s at 476x630 with three heads).  The
 * pipelined rate the benchmark reports (about 1800 frames/s) needs encoder_lanes = 3 and ring_slots = 4 (lanes + 1),
 * which makes the engine use 3 encoder streams + 1 head stream, AND a process that may use five hardware queues:
 * export GPU_MAX_HW_QUEUES=5 before the HIP runtime initialises (the runtime's default of 4 leaves three for the
 * engine beside the default stream's, and the fourth engine stream then shares a queue and serialises; with the
 * default limit the best choice is encoder_lanes = 2, ring_slots = 3: about 1450 frames/s).  The batched
 * configurations (4 or 8 views per step) want encoder_lanes = 2, ring_slots = 3.
 */
#ifndef VPE_H
#define VPE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct vpe_engine vpe_engine;                 /* opaque, owned by the library */

/* Feature handle returned by vpe_encode: which ring slot holds the frame, and the frame's
 * index (0 for the first vpe_encode of the engine, then 1, 2, ...).  A plain value. */
typedef struct { int32_t slot; int32_t reserved; int64_t frame; } vpe_feat;

typedef enum { VPE_OK = 0, VPE_SKIPPED = 1, VPE_BUSY = 2, VPE_EINVAL = -1, VPE_ENOMEM = -2, VPE_ESTALE = -3,
               VPE_EHIP = -4 } vpe_status;
typedef enum { VPE_F32 = 0, VPE_BF16 = 1 } vpe_dtype;
typedef enum { VPE_MLP_GELU = 0, VPE_MLP_SWIGLU = 1 } vpe_mlp;
typedef enum { VPE_HEAD_SEG = 0, VPE_HEAD_DEPTH = 1, VPE_HEAD_DET = 2, VPE_HEAD_DPT = 3 } vpe_head_kind;

enum {
    VPE_FLAG_GRAPHS = 1,     /* replay the encoder and the heads as captured HIP graphs */
    VPE_FLAG_HOST_ONLY = 2,  /* no device at all: calls do the scheduling bookkeeping only (slot ring, rates,
                                staleness, counters); for exercising the host logic on a machine without a GPU */
    VPE_FLAG_WALL_CLOCK = 4, /* vpe_encode stamps each frame with the host's steady clock (seconds since
                                vpe_create), so limits in Hz act on real time without the caller keeping one */
    VPE_FLAG_TIMING = 8      /* record HIP events with timing around every encoder pass and head run, for
                                vpe_stage_times (two more event records per enqueue) */
};

/*
 * Backbone: a DINOv2-style ViT with 14x14 patches (paper, Sec. "Example implementation":
 * the encoder outputs its final features and three evenly spaced intermediate layers).
 *   tokens per image N = 1 + registers + (img_h/14)*(img_w/14): CLS, registers, patches.
 *   taps[k] (1-based, strictly increasing, taps[3] == depth): after block taps[k] the shared
 *   final LayerNorm of the residual stream is written to feature map k of the slot.
 *   dtype: VPE_F32 = fp32 storage and fp32 MFMA arithmetic; VPE_BF16 = bf16 operands with
 *   fp32 accumulation, fp32 residual stream and LayerNorm statistics.
 *   weights: HOST pointer to fp32 values in this order (linear weights [in][out]):
 *     patch_w [dim][3][14][14], patch_b [dim], cls [dim], reg [registers][dim],
 *     pos [1 + patches][dim]  (row 0 is added to CLS, row 1+p to patch p; registers get none),
 *     then per block: ln1_g, ln1_b [dim], qkv_w [dim][3 dim], qkv_b [3 dim]
 *       (columns: queries of all heads, keys, values; head i owns 64 i .. 64 i + 63 of each),
 *       proj_w [dim][dim], proj_b [dim], ls1 [dim], ln2_g, ln2_b [dim],
 *       fc1_w [dim][F], fc1_b [F]  (F = mlp_hidden for GELU; 2 mlp_hidden for SwiGLU: gate half, then linear half),
 *       fc2_w [mlp_hidden][dim], fc2_b [dim], ls2 [dim];
 *     then norm_g, norm_b [dim].
 *   The blob is read during vpe_create only; the caller keeps ownership and may free it after.
 */
typedef struct {
    int32_t dim;          /* = heads * 64 */
    int32_t depth;
    int32_t heads;
    int32_t mlp_hidden;
    int32_t mlp_kind;     /* vpe_mlp */
    int32_t registers;
    int32_t img_h, img_w; /* multiples of 14 */
    int32_t batch;
    int32_t dtype;        /* vpe_dtype */
    int32_t taps[4];
    int32_t ring_slots;   /* >= 1; 2 or more lets encode(f+1) overlap heads(f) */
    int32_t flags;        /* VPE_FLAG_* */
    float   ln_eps;
    int32_t encoder_lanes; /* 1..4 (0 = 1; at most ring_slots): encoder scratch sets and streams; with k >= 2 the
                              encoder passes of k consecutive frames overlap on the GPU -- throughput pipelining,
                              per-frame results are unchanged */
    int32_t head_streams; /* streams the heads are spread over (heaviest head first, onto the least loaded);
                              0 = as many as heads, within the four hardware queues a process gets by default
                              minus the encoder lanes (at least 1).  Heads sharing a stream run in call order */
    int32_t reserved;
    const void* weights;  /* host, fp32 */
    uint64_t weights_bytes;
} vpe_backbone_cfg;

/*
 * Heads (paper, Sec. "Head Module" and "Example implementation"), all reading patch rows of
 * the slot's feature maps as an [img_h/14][img_w/14][dim] channels-last grid:
 *   VPE_HEAD_SEG   linear segmentation: 1x1 conv dim->classes on the final map; bilinear x14
 *                  (half-pixel centres) to img_h x img_w; per-pixel argmax (ties -> lowest).
 *                  weights: seg_w [classes][dim], seg_b [classes].
 *                  outputs: 0 = logits fp32 [B][gh][gw][classes]; 1 = class map u8 [B][img_h][img_w].
 *   VPE_HEAD_DET   dense detection: two parallel 3x3 conv towers dim->channels (+ReLU) on the
 *                  final map, then 1x1 to `classes` logits (class tower) and 4 box offsets (box tower).
 *                  weights: cls_tower_w [ch][dim][3][3], cls_tower_b [ch], box_tower_w, box_tower_b (same
 *                  shapes), cls_w [classes][ch], cls_b, box_w [4][ch], box_b.
 *                  outputs: 0 = fp32 [B][gh][gw][classes + 4] (logits then box); 1 = class map u8 [B][gh][gw].
 *   VPE_HEAD_DEPTH DPT-lite: stage s = 0..3 takes feature map 3 - s: 1x1 conv dim->ch, bilinear to
 *                  2^s x the patch grid, add the previous stage's output, 3x3 conv ch->ch + ReLU, bilinear x2;
 *                  then 1x1 conv ch->1, bilinear to img_h x img_w, ReLU.
 *                  weights: proj{0..3}_w [ch][dim], proj{s}_b [ch] (pairs, s ascending), then
 *                  fuse{0..3}_w [ch][ch][3][3], fuse{s}_b [ch] (pairs), out_w [1][ch], out_b [1].
 *                  outputs: 0 = depth fp32 [B][img_h][img_w].
 *   VPE_HEAD_DPT   the full dense-prediction-transformer depth head (the structure of the DepthAnythingV2 head
 *                  of the paper's example implementation), width F = channels (64, 128, 192 or 256), reassembled
 *                  widths oc_i = (3 F / 4) 2^i; feature map i = 0..3 (shallow to deep) is level i:
 *                    reassemble: 1x1 conv dim->oc_i, then level 0: transposed conv kernel = stride = 4; level 1:
 *                      transposed conv kernel = stride = 2; level 2: nothing; level 3: 3x3 conv stride 2 padding 1;
 *                      then 3x3 conv oc_i->F without bias, giving l_i on the 4x, 2x, 1x, ceil(1/2)x patch grid;
 *                    fusion, k = 3..0: s_3 = l_3, s_k = path_{k+1} + unit(l_k); path_k = 1x1 conv F->F of the
 *                      bilinear resize with aligned corners of unit(s_k) to level k-1's grid (k = 0: to twice its
 *                      own); unit(x) = x + conv3x3(ReLU(conv3x3(ReLU(x)))), both with bias;
 *                    output: 3x3 conv F->F/2 of path_0, aligned-corner bilinear to img_h x img_w, 3x3 conv
 *                      F/2->32 + ReLU, 1x1 conv 32->1, ReLU.
 *                  weights: proj{0..3}_w [oc_i][dim], proj{i}_b (pairs); up0_w [oc_0][oc_0][4][4] (input channel
 *                  first), up0_b; up1_w [oc_1][oc_1][2][2], up1_b; down3_w [oc_3][oc_3][3][3], down3_b;
 *                  rn{0..3}_w [F][oc_i][3][3]; for k = 3, 2, 1, 0: (k < 3: unit a: c1_w [F][F][3][3], c1_b, c2_w,
 *                  c2_b,) unit b: c1_w, c1_b, c2_w, c2_b, out_w [F][F], out_b; head1_w [F/2][F][3][3], head1_b;
 *                  head2_w [32][F/2][3][3], head2_b; head3_w [1][32], head3_b [1].
 *                  outputs: 0 = depth fp32 [B][img_h][img_w].
 *   every_n >= 1: the head runs on frame f iff f % every_n == 0 (paper, Sec. "Dynamic Frequency Control").
 */
typedef struct {
    int32_t kind;         /* vpe_head_kind */
    int32_t classes;      /* seg: C; det: number of object classes; depth, dpt: ignored */
    int32_t channels;     /* det / depth / dpt hidden width (multiple of 64; dpt: at most 256); seg: ignored */
    int32_t every_n;
    const void* weights;  /* host, fp32 */
    uint64_t weights_bytes;
} vpe_head_cfg;

/* Device bytes the engine needs for weights, scratch, the feature ring and head outputs (paper, Sec. "Memory
 * Management": buffer sizes are fixed by the configuration and allocated once at start-up).
 * Returns 0 and sets *bytes, or VPE_EINVAL. */
int vpe_workspace_bytes(const vpe_backbone_cfg* cfg, const vpe_head_cfg* heads, int n_heads, uint64_t* bytes);

/* Build an engine.  workspace: DEVICE memory of at least vpe_workspace_bytes, 256-byte aligned,
 * owned by the caller and kept alive until vpe_destroy (lets the caller's allocator own all
 * device memory); NULL makes the library allocate it once with hipMalloc.  Uploads and re-lays
 * the weights, zeroes padding, creates streams and events.  After this returns the engine
 * never allocates device memory (paper, Sec. "Memory Management": preallocate at start-up). */
int vpe_create(const vpe_backbone_cfg* cfg, const vpe_head_cfg* heads, int n_heads,
               void* workspace, uint64_t workspace_bytes, vpe_engine** out);

/* The foundation module's step (paper, Sec. "Foundation Module": input -> foundation model -> middle buffer,
 * and Sec. "Data Flow": the middle buffer is a circular buffer that overwrites its oldest entry).
 * Encode one batch: images = DEVICE fp32 [batch][3][img_h][img_w], already normalised; it must
 * stay valid until the enqueued work has run.  Picks ring slot frame % ring_slots, waits (on
 * the GPU) for heads still reading that slot, runs the encoder, and returns the handle.
 * Errors: VPE_EINVAL (null engine / images / out), VPE_EHIP (a launch failed). */
int vpe_encode(vpe_engine* e, const float* images, void* stream, vpe_feat* out);

/* Camera-frame transform in front of vpe_encode (paper, Sec. "Transforms": the pre-processing adapter between
 * user data and the foundation model -- type conversion, resizing, normalisation -- runs on the GPU).
 *   frames: DEVICE uint8 [batch][src_h][src_w][3], interleaved RGB;  images: DEVICE fp32 [batch][3][dst_h][dst_w];
 *   images[c] = (bilinear(frames[..., c] / 255 -> dst_h x dst_w) - mean[c]) / std[c], half-pixel centres, no
 *   antialiasing filter (the paper does not say how its 1920x1080 frames reach the model's resolution);
 *   mean, std: HOST, 3 floats each, std > 0.
 * Needs no engine; only enqueues (stream NULL = the default stream); the caller owns both buffers.  Returns
 * VPE_EINVAL on null pointers, non-positive sizes or std <= 0, VPE_EHIP on a launch failure. */
int vpe_preprocess_u8(const uint8_t* frames, int batch, int src_h, int src_w, float* images, int dst_h, int dst_w,
                      const float mean[3], const float std[3], void* stream);

/* The engine-owned stream that the next vpe_encode / vpe_encode_at with stream == NULL will run on (one per
 * encoder lane, taken in turn).  Work the caller enqueues on it first -- vpe_preprocess_u8, a host-to-device
 * copy of the frame -- is ordered before that encode without an event and without another stream competing
 * for a hardware queue.  Borrowed: do not destroy it.  host-only engines return NULL in *stream. */
int vpe_next_encode_stream(vpe_engine* e, void** stream);

/* As vpe_encode, for a frame captured at time t_seconds (any monotonic clock of the caller's: a camera
 * timestamp, or frame index / frame rate).  The time is kept with the frame and is what per-head limits in
 * Hz (vpe_set_head_rate_hz) are measured against; frames encoded with vpe_encode carry no time and are
 * not limited in Hz, unless the engine was created with VPE_FLAG_WALL_CLOCK.  t_seconds must not decrease from one frame to the next (VPE_EINVAL). */
int vpe_encode_at(vpe_engine* e, const float* images, void* stream, double t_seconds, vpe_feat* out);

/* A head module's step (paper, Sec. "Head Module": each head reads the middle buffer asynchronously, by
 * reference, runs its model and leaves its post-processed result in its output buffer; Sec. "Dynamic Frequency
 * Control" for the rate).  Enqueues head `head` on the features of frame fh, in place, on `stream` (NULL = the
 * head's own stream) after the frame's encoder pass and the head's previous run.  Returns VPE_SKIPPED when
 * fh.frame % every_n != 0 or a limit in Hz says the frame is not due, VPE_ESTALE when the slot has been reused by
 * a later frame, VPE_EINVAL for an unknown head or a handle this engine did not produce, VPE_EHIP. */
int vpe_run_head(vpe_engine* e, int head, vpe_feat fh, void* stream);

/* vpe_run_head for callers that cannot allocate device memory or let a library do so on their behalf: tight
 * serving loops, harnesses that forbid hipMalloc, code that must not trigger the lazy graph instantiation of
 * vpe_run_head.  Same arguments, checks, return values, scheduling and outputs (the head's own output buffers, read
 * with vpe_head_output); the difference is where the run's intermediate buffers live and how it is launched:
 *   - they are taken from a file-scope device array inside the library (8 MiB, one copy per GPU, held until the
 *     process ends) instead of from the engine's workspace;
 *   - the head's kernels are always launched one by one (never as a graph replay, even with VPE_FLAG_GRAPHS), and
 *     the call performs no hipMalloc / hipFree / graph instantiation.
 * Supported heads: VPE_HEAD_SEG (needs none), VPE_HEAD_DET (batch * patches * 2 channels elements), VPE_HEAD_DEPTH
 * (about 129 * batch * patches * channels elements); a head whose buffers exceed 8 MiB and VPE_HEAD_DPT are
 * refused with VPE_EINVAL and a message that states both sizes.  Nothing in the array needs clearing (a run writes
 * every element before it reads it), and it keeps the last run's contents.  All calls on one GPU share the array:
 * two vpe_run_head_static runs that overlap on a GPU (different heads, engines or streams) race -- order them
 * on one stream or wait for the first (vpe_head_done / vpe_wait_head) before starting the next.  The engine's GPU
 * must be the current device (VPE_EINVAL otherwise). */
int vpe_run_head_static(vpe_engine* e, int head, vpe_feat fh, void* stream);

/* Has the encoder finished writing this frame's features?  VPE_OK = yes, VPE_BUSY = still executing,
 * VPE_ESTALE = the slot has been taken by a later frame (no error message is set for these three).  A producer
 * that must not run further ahead of the device than the ring is long polls the handle it got `ring_slots - 1`
 * frames ago.  Never blocks. */
int vpe_frame_ready(vpe_engine* e, vpe_feat fh);

/* Run head `head` on the NEWEST frame whose features are complete, the way the paper's decentralised modules do (Sec.
 * "Decentralization", "Data Flow": modules never wait for each other, a circular buffer overwrites its oldest
 * entry, so a slow head works on the freshest features and loses the frames in between).  In order:
 *   VPE_SKIPPED  no frame has been encoded since this head last asked (through this call or vpe_run_head);
 *   VPE_BUSY     the head's previous run is still executing on the device: nothing is queued behind it, call
 *                again later (never returned by host-only engines);
 *   VPE_SKIPPED  none of the frames encoded since then, and still in the ring, has finished on the device;
 *   VPE_SKIPPED  the newest frame is fewer than every_n frames after the head's last run, or the limit in Hz
 *                does not allow it yet;
 *   VPE_OK       the run was enqueued; *ran_on (may be NULL) receives the frame's handle.
 * Frames between the last one the head asked about and the one it takes now are counted as missed (see
 * vpe_head_counters).  Never blocks the host.  While the head reads a slot, an encode into that slot waits on the
 * device (not on the host): size the ring so that ring_slots frame periods exceed the slowest head's run time. */
int vpe_run_head_latest(vpe_engine* e, int head, void* stream, vpe_feat* ran_on);

/* Per-head counters, all since vpe_create:
 *   out[0] runs, out[1] skips (not due), out[2] missed: frames passed over by vpe_run_head_latest taking a newer
 *   one, out[3] overflow: frames overwritten in the ring before this head had asked about them or a later frame
 *   (the signal that the consumer does not keep pace with the producer; paper, Sec. "Data Flow"),
 *   out[4] busy returns, out[5] frame of the last run (-1 = none), out[6] newest frame asked about (-1 = none),
 *   out[7] reserved (0). */
int vpe_head_counters(vpe_engine* e, int head, int64_t out[8]);

/* Change a head's rate at run time (paper, Sec. "Dynamic Frequency Control": the rate of every head can be
 * adjusted while the engine runs): the head runs on frame f iff f % every_n_frames == 0.  Takes effect from the
 * next vpe_run_head.  every_n_frames < 1 or an unknown head -> VPE_EINVAL. */
int vpe_set_head_rate(vpe_engine* e, int head, int every_n_frames);

/* Upper limit on a head's rate in runs per second of frame time (paper, Sec. "Dynamic Frequency Control"
 * and Appendix "Rate-Limiting Experiment": each head's rate can be set at run time, and over 300 frames at
 * 30 Hz the delivered counts stay within one frame of rate x duration); 0 = no limit.
 * The head keeps a due time: a frame stamped t (vpe_encode_at) is processed iff t >= due (less a millionth
 * of a period, for rounding), and the due time then advances by one period 1 / max_hz (it accumulates, so a limit that is not
 * a divisor of the input rate is met on average: over any span the number of runs differs from
 * span * max_hz by at most one); after a gap of more than a period the due time restarts from the
 * frame's time.  A frame that is not due returns VPE_SKIPPED, like the frame divider, which still applies
 * (both must pass).  Takes effect from the next vpe_run_head; max_hz < 0 or not finite -> VPE_EINVAL. */
int vpe_set_head_rate_hz(vpe_engine* e, int head, double max_hz);

/* The middle buffer's labelled entries (paper, Sec. "Data Flow": features are kept as named tensors and handed
 * over by reference; Sec. "Memory Management": no copies between modules).  Borrowed DEVICE pointer to feature
 * map `tap` (0..3 = after blocks taps[0..3], 3 = the final tokens) of a frame: [batch][N][dim] in the engine's
 * dtype.  Valid until the slot is reused (VPE_ESTALE once it has been); VPE_EINVAL for a bad tap or handle. */
int vpe_feat_view(vpe_engine* e, vpe_feat fh, int tap, const void** dev_ptr, int64_t shape[3]);

/* A head's output buffer (paper, Sec. "Head Module": post-processed results are placed in an output buffer).
 * Borrowed DEVICE pointer to output `which` of a head (see vpe_head_cfg); shape is padded with 1s to four
 * entries.  One instance per head: contents are those of the head's most recent run once vpe_head_done says it
 * has finished, and the head's next run overwrites them (a consumer that needs a result for longer copies it,
 * or orders its own stream after the run with the stream argument of vpe_run_head).  VPE_EINVAL if the head
 * has no such output. */
int vpe_head_output(vpe_engine* e, int head, int which, const void** dev_ptr, int64_t shape[4]);

/* Has head `head` finished its most recent run (paper, Sec. "Head Module": consumers take results from the
 * head's output buffer; Sec. "Decentralization": nobody blocks on anybody)?  VPE_OK = yes (or it never ran),
 * VPE_BUSY = still executing.  Never blocks.  vpe_wait_head blocks the host until that run has finished (that
 * head only: other heads and the encoder keep going). */
int vpe_head_done(vpe_engine* e, int head);
int vpe_wait_head(vpe_engine* e, int head);

/* Block until everything enqueued through THIS engine has finished (its encoder passes and head runs, on
 * whichever streams they were put); other work of the process on the device is not waited for. */
int vpe_sync(vpe_engine* e);

/* Counters (paper, Appendix "Rate-Limiting Experiment": delivered runs per head): frames encoded, and per head
 * (up to n entries) how often it ran / was skipped.  Any output pointer may be NULL. */
int vpe_stats(vpe_engine* e, int64_t* frames, int64_t* head_runs, int64_t* head_skips, int n);

/* Device time of the most recent encoder pass and of each head's most recent run, in milliseconds (paper, Sec.
 * "Example implementation" reports per-head inference times): *encode_ms and head_ms[0 .. n-1]; -1 where nothing
 * has run yet or the run is still executing.  Needs VPE_FLAG_TIMING (else VPE_EINVAL).  Never blocks.  The span
 * is from the start of the stage's first kernel to the end of its last on its stream; under load it includes
 * the time the stage's kernels shared the device with other stages. */
int vpe_stage_times(vpe_engine* e, float* encode_ms, float* head_ms, int n);

/* Timing aid for benchmarks and counter passes (not part of the data path): waits until the engine is idle, then
 * enqueues `reps` repetitions of one internal kernel family on the encoder stream with HIP events around them and
 * returns the mean milliseconds per launch.  It overwrites scratch of encoder lane 0 and of the depth head only
 * (buffers that the next encode / head run rewrites before reading); feature slots and head outputs are untouched.
 * which: 0 = the fused-QKV GEMM of block 0 on the current activations, 1 = the attention
 * kernel of block 0, 2 = LayerNorm, 3 = the depth head's largest 3x3 convolution (last fusion stage; needs a
 * depth head), 4 = the resample-and-add kernel that writes that convolution's input (needs a depth head),
 * 5 = the out-projection GEMM of block 0 (LayerScale + residual epilogue), 6 = its fc1 GEMM (LayerNorm folded in,
 * GELU or SwiGLU epilogue), 7 = its fc2 GEMM (LayerScale + residual epilogue), 8 = a stand-alone activation pass over
 * the MLP hidden buffer (the bandwidth-bound kernel the fused epilogue replaces), 9 = the fc1 GEMM with a plain store
 * (no activation; mlp_hidden columns): 9 + 8 against 6 is what the fusion saves.
 * Also reports the algorithmic flops and bytes of one launch. */
int vpe_time_kernel(vpe_engine* e, int which, int reps, float* ms_per_launch, double* flops, double* bytes);

/* Message of the most recent failure of a call on this engine (engine may be NULL: the last failure of a call
 * that had no engine, on this thread).  Borrowed; valid until the next failing call. */
const char* vpe_last_error(vpe_engine* e);
/* Waits for the device, destroys streams, events and graphs, frees the workspace if the library allocated it. */
void vpe_destroy(vpe_engine* e);

#ifdef __cplusplus
}
#endif
#endif /* VPE_H */
