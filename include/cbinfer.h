/*
 * cbinfer.h -- C ABI of the MI355X change-based convolution library.
 *
 * The library evaluates a fixed convolutional network on the frames of a static-camera
 * video, recomputing per frame and per convolution layer only the output positions whose
 * filter support saw an input change (CBinfer, arXiv 1704.04313, Section 3).
 *
 * Conventions
 *   - C99, plain pointers and sizes; no C++ types, no exceptions cross this boundary.
 *   - "HOST" / "DEVICE" on a pointer says which memory it must point to.
 *   - Frames and outputs are planar [n_streams][C][H][W] float32 (Section 3: the image matrix
 *     X is built from x(k, j+y_o, i+x_o)); weights are [cout][cin][kh][kw], the row layout of
 *     the filter matrix K (Section 3).
 *   - Positions in index lists are int32 linear indices  stream*H*W + y*W + x  of the map
 *     they refer to, strictly ascending.
 *   - Every function returning int returns CBINFER_OK (0) or a negative error code and
 *     stores a message readable with cbinfer_last_error() (thread-local).
 *   - Nothing here falls back to a CPU implementation: without a usable HIP device
 *     cbinfer_create fails with CBINFER_EDEVICE.
 */
#ifndef CBINFER_H
#define CBINFER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cbinfer_state cbinfer_state; /* opaque; owns all per-layer state */

enum {
    CBINFER_OK = 0,
    CBINFER_EINVAL = -1,       /* bad argument or inconsistent network description */
    CBINFER_EUNSUPPORTED = -2, /* valid but not implemented (size limits, layer combinations) */
    CBINFER_ENOMEM = -3,       /* device allocation failed or caller workspace too small */
    CBINFER_EDEVICE = -4,      /* a HIP call failed; the state must be destroyed */
    CBINFER_ESTATE = -5        /* call not valid in the current state (e.g. no frame yet) */
};

enum { CBINFER_OP_CONV = 0, CBINFER_OP_MAXPOOL = 1 };
enum { CBINFER_F32 = 0, CBINFER_BF16 = 1 };

/* cbinfer_network.flags */
enum {
    /* Which value the stored "previous input" keeps at positions that were NOT flagged.
     * 0: the previous frame's layer input at every position, the x^(t-1) of the change
     *    detection formula (Section 3.1).  1: only flagged positions are refreshed. */
    CBINFER_FLAG_HOLD_REFERENCE = 1u,
    /* Write the index lists of every layer (changed inputs, outputs to update, pooled positions
     * -- the lists of Section 3.1) in every frame, with the dilation and extraction kernels, also
     * for maps small enough for the multiplication kernel to pick its positions from the update
     * map itself.  Results are the same; cbinfer_read_list / cbinfer_layer_counts then find the
     * lists ready instead of extracting them on demand, at the price of two or three more
     * launches per layer and frame. */
    CBINFER_FLAG_LISTS_EVERY_FRAME = 2u,
    /* Throughput mode: consecutive frames may overlap on the device.  The library enqueues frames
     * alternately on two streams of its own (default priority) and keeps two sets of per-frame
     * scratch (change maps, index lists, partial sums); events make every kernel that overwrites a
     * stored map of Section 3.2 wait for the previous frame's kernels that still read it, so each
     * frame sees exactly the state the frame before it left -- results are the same as without the
     * flag.  What changes is when a frame's output is complete for the caller: cbinfer_process_frame
     * no longer orders the state's stream behind the frame; cbinfer_flush does (all frames so far),
     * and so does every introspection call.  Work pending on the state's stream when a frame is
     * passed in still comes first; frame and output buffers must stay untouched until a flush has
     * covered their frame.  Costs a second scratch set (cbinfer_workspace_bytes says how much).
     * Networks of fewer than three operations ignore the flag (nothing to overlap). */
    CBINFER_FLAG_PIPELINE_FRAMES = 4u
};

/* One operation of the network, in execution order. */
typedef struct {
    int32_t kind;      /* CBINFER_OP_CONV or CBINFER_OP_MAXPOOL */
    int32_t cin, cout; /* CONV: channel counts.  MAXPOOL: ignored */
    int32_t kh, kw;    /* CONV: filter size.  MAXPOOL: window (kh == kw == stride, 2 supported) */
    int32_t stride;    /* CONV: >= 1 */
    int32_t pad;       /* CONV: zero padding on every side, 0 <= pad < min(kh, kw).  MAXPOOL: 0 */
    int32_t relu;      /* CONV: apply max(0, .) in the output update (Section 3.1, "Output Updating") */
    int32_t dense;     /* CONV: 1 = recompute every position every frame (the paper kept its two
                          pixel-classification layers dense, Section 4.2) */
    int32_t propagate; /* CONV behind the first: 1 = no change detection of its own; every input position the
                          op before it recomputed counts as changed (the worst-case change propagation that
                          Section 4.7 compares per-layer detection with).  Not together with dense */
    float threshold;   /* CONV: change-detection threshold tau of this layer (Section 3.3);
                          negative = use the global threshold given to cbinfer_create */
    const void *weight; /* HOST, [cout][cin][kh][kw] float32, read during cbinfer_create only */
    const float *bias;  /* HOST, [cout] float32 or NULL for zeros, read during cbinfer_create only */
} cbinfer_layer;

typedef struct {
    int32_t n_layers;
    const cbinfer_layer *layers; /* HOST, read during cbinfer_create only */
    int32_t in_c, in_h, in_w;    /* frame shape per stream */
    int32_t n_streams;           /* >= 1 independent cameras processed together; each has its own
                                    state; index lists are concatenated in stream order */
    int32_t dtype;               /* storage type of the library's internal maps and filter matrices:
                                    CBINFER_F32, or CBINFER_BF16 (values rounded to nearest even, float32
                                    accumulation); frames, outputs, bias and thresholds are float32 either way */
    uint32_t flags;              /* CBINFER_FLAG_* */
    void *stream;                /* hipStream_t all work is enqueued on (NULL = default stream) */
    void *workspace;             /* DEVICE memory for all state and scratch, 256-byte aligned, or
                                    NULL to let the library allocate (and own) it */
    size_t workspace_bytes;      /* size of workspace; ignored when workspace is NULL */
} cbinfer_network;

/* Bytes of device memory a state for this network needs; 0 if the description is invalid
 * (cbinfer_last_error says why).  Touches no device. */
size_t cbinfer_workspace_bytes(const cbinfer_network *net);

/* Build the per-layer state of Section 3.2 (previous input and previous output of every
 * convolution layer) plus change maps and index lists, and upload the filter matrices.
 * threshold: global tau (>= 0, finite) for layers whose own threshold is negative.
 * Returns NULL on error.  The first frame after create is evaluated densely. */
cbinfer_state *cbinfer_create(const cbinfer_network *net, float threshold);

/* For callers that cannot allocate device memory (set-up code of a pipeline that is later replayed
 * from a HIP graph, serving loops and harnesses that forbid hipMalloc): cbinfer_create without any
 * device allocation and without a caller workspace.  All state and scratch of the network live in
 * a device array of CBINFER_STATIC_WORKSPACE_BYTES that is part of the library itself; every GPU
 * the library is loaded on holds one such array from load time until the process ends.
 * net->workspace and net->workspace_bytes are ignored.  The state is created on the current device.
 * Errors (NULL returned, message in cbinfer_last_error): everything cbinfer_create rejects;
 * CBINFER_ENOMEM if the network needs more than CBINFER_STATIC_WORKSPACE_BYTES
 * (cbinfer_workspace_bytes tells how much it needs; the 320x240 scene-labeling network fits, the
 * 1280x720 and 64-stream workloads do not); CBINFER_ESTATE while another state created by this
 * call is still alive on the same device: there is one array per device, so at most one such
 * state per device may exist at a time, and two processes' worth of frames must not be
 * interleaved through it.  The array keeps the previous state's contents; this call clears the
 * part it uses.  cbinfer_destroy releases the array for the next state (and frees nothing).
 * Everything else (cbinfer_process_frame, reset, introspection) works as for any other state. */
#define CBINFER_STATIC_WORKSPACE_BYTES (64u << 20)
cbinfer_state *cbinfer_create_static(const cbinfer_network *net, float threshold);
size_t cbinfer_static_workspace_bytes(void); /* CBINFER_STATIC_WORKSPACE_BYTES of the loaded build */

/* Process one frame: for every convolution layer, change detection against the stored
 * previous input, change-index extraction, dilation by the filter support into the list of
 * outputs to recompute, reduced matrix multiplication over those columns only, and the
 * output update with bias and ReLU (Section 3.1); changes are carried through max-pooling
 * by recomputing only the pooled positions whose window was updated.
 * frame_dev: DEVICE, [n_streams][in_c][in_h][in_w] float32.
 * out_dev:   DEVICE, [n_streams][cout_last][Ho][Wo] float32; receives the complete stored
 *            output of the last operation.
 * Asynchronous: all work is enqueued on the state's stream and nothing is allocated; the host
 * does not wait for the device -- except while per-step timing is enabled
 * (cbinfer_set_profiling), when the call returns only after the frame has run and its kernel
 * times have been collected.  Both buffers must stay valid until that work has run. */
int cbinfer_process_frame(cbinfer_state *s, const void *frame_dev, void *out_dev);

/* With CBINFER_FLAG_PIPELINE_FRAMES: make the state's stream wait for the frame enqueued last (and
 * with it for all before), so that work enqueued on it afterwards sees their outputs.  Without the
 * flag: nothing to do.  Does not block the host. */
int cbinfer_flush(cbinfer_state *s);

/* Forget the video history: the stored previous inputs and outputs of Section 3.2 count as
 * absent, so the next frame is evaluated densely like the first one (all positions flagged, identity
 * lists).  Frees nothing, waits for nothing. */
int cbinfer_reset(cbinfer_state *s);

/* Waits for the stream, then releases everything the library allocated.  NULL is a no-op. */
void cbinfer_destroy(cbinfer_state *s);

const char *cbinfer_last_error(void); /* never NULL */

/* 1: per-frame dense evaluation of every layer through the same kernels with the identity
 * index list and no change detection (the dense baseline the speed-up is measured against;
 * Section 3.1: the reduced multiplication is at worst the full-frame convolution).
 * 0: change-based evaluation.  Switching also resets the history. */
int cbinfer_set_mode(cbinfer_state *s, int force_dense);

/* ---- introspection (each call waits for the stream first) ------------------------------ */

/* Shape of operation `layer`'s output map, per stream. */
int cbinfer_layer_shape(cbinfer_state *s, int layer, int32_t *c, int32_t *h, int32_t *w);

/* Lengths of the index lists of Section 3.1 ("Change Indexes Extraction") for operation `layer`
 * in the last frame: changed input positions (CONV; -1 for MAXPOOL) and output positions
 * recomputed (CONV: the dilated change map's positions; MAXPOOL: pooled positions recomputed). */
int cbinfer_layer_counts(cbinfer_state *s, int layer, int64_t *n_changed, int64_t *n_update);

enum { CBINFER_LIST_CHANGED = 0, CBINFER_LIST_UPDATE = 1, CBINFER_LIST_POOLED = 2 };
/* Copy an index list of the last frame (Section 3.1, "Change Indexes Extraction") to HOST memory.
 * CONV: CHANGED = input positions whose change exceeded tau (first formula of Section 3.1),
 * UPDATE = output positions recomputed (the dilated change map, second formula), POOLED = the
 * positions of the pooling operation directly behind this layer that were recomputed (an error if
 * there is none).  MAXPOOL: UPDATE only (the same list as the convolution's POOLED).
 * *n receives the list length; at most cap entries are written. */
int cbinfer_read_list(cbinfer_state *s, int layer, int which, int32_t *host, int64_t cap, int64_t *n);

enum { CBINFER_MAP_REFERENCE = 0, CBINFER_MAP_OUTPUT = 1 };
/* Copy one of the per-layer buffers of Section 3.2 to HOST memory as planar float32
 * [n_streams][C][H][W] (bfloat16 storage is widened).  REFERENCE: the stored previous input of a
 * CONV layer.  OUTPUT: the stored output map.
 * count = number of floats `host` can take; must equal the map size. */
int cbinfer_read_map(cbinfer_state *s, int layer, int which, float *host, size_t count);

/* ---- per-step timing -------------------------------------------------------------------- */

enum {
    CBINFER_STEP_DETECT = 0,  /* change detection + update of the stored previous input */
    CBINFER_STEP_DILATE = 1,  /* change map -> map of outputs to update (and of pooled outputs) */
    CBINFER_STEP_COMPACT = 2, /* maps -> ascending index lists and counts */
    CBINFER_STEP_GEMM = 3,    /* gathered matrix generation + multiplication + output update */
    CBINFER_STEP_POOL = 4,    /* max-pooling at the listed pooled positions */
    CBINFER_STEP_OUTPUT = 5,  /* copy of the last stored map to the caller's buffer (layer = last) */
    CBINFER_STEP_COUNT = 6
};

/* enable != 0: bracket every kernel launch of later frames with HIP events on the state's
 * stream (slows frames down a little; meant for measurement runs).  Clears the totals. */
int cbinfer_set_profiling(cbinfer_state *s, int enable);

/* Total kernel time in milliseconds and number of launches recorded since profiling was
 * enabled, for one step of one operation. */
int cbinfer_read_profile(cbinfer_state *s, int layer, int step, double *ms_total, int64_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* CBINFER_H */
