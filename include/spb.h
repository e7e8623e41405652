/*
 * spb.h - C ABI of the Structured Partial Backpropagation (SPB) worker step.
 *
 * One worker's training step as the paper states it (Sec. 2): run the complete
 * forward pass to the loss, then backpropagate over a fixed suffix of the
 * network, starting at the output layer, and hand over the gradients of that
 * suffix only.  Layers below the cut get no input gradient, no weight gradient
 * and no saved activation (Sec. 1: outputs of layers that take no part in the
 * backward pass need not be kept).
 *
 * A model is an ordered list of units; the backward pass may stop only between
 * units.  L = number of units.  Depth k = number of units, counted from the
 * output end, that are backpropagated: k = 0 computes no gradient, k = L is
 * ordinary backpropagation.
 *
 * Conventions
 *   - Every call returns 0 (SPB_OK) or a negative error code; spb_last_error()
 *     gives the message of the calling thread's last failure.  Argument errors
 *     are found on the host before anything is enqueued.
 *   - The library allocates no device memory.  Parameters, gradient buffers,
 *     inputs, labels and one workspace are DEVICE pointers owned by the caller
 *     and must stay alive until the stream work that uses them has completed.
 *     Parameters stay resident on the device between calls (cf. Sec. 3, keeping
 *     model parameters in GPU memory across task switches).
 *   - Work is enqueued on the caller's stream (a hipStream_t passed as void*);
 *     calls return without waiting for the device and may be captured into a
 *     HIP graph.  Calls on one model must not overlap in time.
 *   - A model owns one more HIP stream and a few events (no device memory),
 *     created by its first spb_forward outside a graph capture and released by
 *     spb_model_destroy.  spb_backward_truncated runs weight-gradient kernels on
 *     it beside the input-gradient chain; it first makes that stream wait for the
 *     caller's and, before it returns, makes the caller's stream wait for it, so
 *     to the caller everything is ordered on the stream that was passed.  While
 *     that stream is being captured, and while kernel timing is on, the extra
 *     stream is not used.  Results are the same bits in every case.
 *   - All matrices are row-major.  Activations of perceptrons are
 *     [batch, features].
 *   - A model needs a GPU; there is no host fallback.
 */
#ifndef SPB_H
#define SPB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPB_OK 0
#define SPB_ERR_INVALID_ARG (-1) /* null pointer, bad shape, misaligned buffer */
#define SPB_ERR_DEPTH_RANGE (-2) /* k < 0 or k > L */
#define SPB_ERR_STATE (-3)       /* backward without forward, or deeper than the forward stashed for */
#define SPB_ERR_WORKSPACE (-4)   /* workspace too small or misaligned */
#define SPB_ERR_HIP (-5)         /* the HIP runtime refused a launch */
#define SPB_ERR_UNSUPPORTED (-6) /* model family not built into this library */

#define SPB_FAMILY_MLP 0               /* Linear(+ReLU) units, softmax cross-entropy on the last */
#define SPB_FAMILY_RESNET_BASIC 1      /* stem | basic residual blocks | pooled classifier */
#define SPB_FAMILY_RESNET_BOTTLENECK 2 /* stem | bottleneck residual blocks | pooled classifier */
#define SPB_FAMILY_ENCODER 3           /* embedding | pre-LN Transformer layers | masked-token head */

#define SPB_DTYPE_F32 0
#define SPB_DTYPE_BF16 1 /* bfloat16 storage, float32 accumulation */
#define SPB_DTYPE_I32 2

#define SPB_MAX_DIMS 64
#define SPB_MAX_STAGES 8
#define SPB_NAME_LEN 48

typedef struct spb_model spb_model;

/* Shape of a model.  Only the fields of the chosen family are read. */
typedef struct spb_model_desc {
  int32_t family; /* SPB_FAMILY_* */
  int32_t dtype;  /* SPB_DTYPE_F32 or SPB_DTYPE_BF16: storage type of parameters, inputs, activations */
  int32_t batch;  /* samples per step */
  /* MLP: n_dims widths, input first; unit i is Linear dims[i] -> dims[i+1]; ReLU after all but the last */
  int32_t n_dims;
  int32_t dims[SPB_MAX_DIMS];
  /* residual CNNs: NHWC images, stem conv (+ optional 3x3/2 max-pool), stages of blocks, classes */
  int32_t image_h, image_w, image_c;
  int32_t stem_kernel, stem_stride, stem_pad, stem_pool, stem_width;
  int32_t n_stages;
  int32_t stage_blocks[SPB_MAX_STAGES];
  int32_t stage_widths[SPB_MAX_STAGES];
  int32_t classes;
  /* encoder */
  int32_t seq, layers, hidden, heads, ffn, vocab, loss_rows;
} spb_model_desc;

/* One parameter tensor of a model. */
typedef struct spb_tensor_info {
  char name[SPB_NAME_LEN]; /* e.g. "fc3.weight" */
  int32_t unit;            /* owning unit, 0 = input end */
  int32_t dtype;           /* storage type of the parameter; its gradient is always float32 */
  int32_t ndim;
  int64_t shape[4];
  int64_t numel;
} spb_tensor_info;

/* One gradient buffer produced by a truncated backward pass. */
typedef struct spb_grad_view {
  int32_t param_index; /* index into spb_param_info */
  int32_t unit;
  void* data;          /* device pointer, float32, the parameter's shape, dense row-major */
  int64_t numel;
} spb_grad_view;

/* Per-kernel timing record (see spb_set_kernel_timing). */
typedef struct spb_kernel_time {
  char name[SPB_NAME_LEN]; /* kernel class; matrix products carry their shape: "gemm_bf16_wgrad 1024x1024x256" */
  int64_t launches;
  double total_ms; /* sum of HIP-event durations of those launches */
  double flops;    /* algorithmic floating-point operations of those launches (2*M*N*K per product) */
  double bytes;    /* algorithmic bytes: each operand read once, each result written once */
} spb_kernel_time;

/* Message of the calling thread's most recent failed call ("" if none).  Host pointer, owned by the library. */
const char* spb_last_error(void);

/* Create the host-side description of a model (unit list, parameter list, buffer plan).
 * desc: host pointer, copied.  out: receives a handle owned by the library until spb_model_destroy.
 * Errors: INVALID_ARG (null, non-positive sizes, feature widths that are not a multiple of 16 bytes
 * except the last), UNSUPPORTED. */
int spb_model_create(const spb_model_desc* desc, spb_model** out);
int spb_model_destroy(spb_model* m);

/* L, the number of units (the layer count L of Sec. 2, counted in units, the granularity of the cut). */
int spb_num_units(const spb_model* m, int32_t* n_units);

/* Parameter list, unit order, input end first. */
int spb_param_count(const spb_model* m, int32_t* n_params);
int spb_param_info(const spb_model* m, int32_t index, spb_tensor_info* out);

/* Bind device buffers.  ptrs: host array of n device pointers, n = spb_param_count; entry i holds
 * parameter i (model dtype, dense row-major) or its gradient buffer (float32, same shape).  Buffers must
 * be 16-byte aligned.  Gradient entries of parameters that no later call backpropagates may be NULL. */
int spb_bind_params(spb_model* m, void* const* ptrs, int32_t n);
int spb_bind_grads(spb_model* m, void* const* ptrs, int32_t n);

/* Bytes of workspace a forward pass that stashes for depth k needs.  Non-decreasing in k: below the
 * cut only two ping-pong activation buffers exist; above it every activation the top k units'
 * backward pass reads is kept (Sec. 1, Table 1's peak-memory column).  Errors: DEPTH_RANGE. */
int spb_workspace_size(const spb_model* m, int32_t k, size_t* bytes);

/* Full forward pass to the loss (Sec. 2: every worker runs the whole forward pass), keeping only what a
 * backward pass of depth <= stash_depth_k will read.
 *   x          device, model dtype: [batch, dims[0]] (MLP), NHWC images (CNN); int32 token ids [batch, seq]
 *              in [0, vocab) (encoder).  Not copied: a backward pass of full depth (k = L) reads x again in every
 *              family (the lowest unit's weight gradient needs its input; the encoder re-reads the ids), so x,
 *              like labels and loss_rows, must stay unchanged until the matching backward call has completed.
 *   labels     device, int32, one class index per loss row, each in [0, classes)
 *   loss_rows  device, int32: the loss_rows distinct positions in [0, batch * seq) that carry a loss
 *              (encoder, read again by the backward pass); NULL otherwise
 *   workspace  device, 256-byte aligned, >= spb_workspace_size(stash_depth_k) bytes; holds the stash
 *              until the matching backward call has completed
 *   loss_out   device, one float32: mean softmax cross-entropy over the loss rows
 * Errors: INVALID_ARG, DEPTH_RANGE, STATE (parameters not bound), WORKSPACE, HIP. */
int spb_forward(spb_model* m, const void* x, const int32_t* labels, const int32_t* loss_rows,
                int32_t stash_depth_k, void* workspace, size_t workspace_bytes, float* loss_out,
                void* stream);

/* The same forward pass for callers that cannot allocate and have no workspace to hand over (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the workspace is a device array of
 * SPB_STATIC_WORKSPACE_BYTES that the library holds itself (one copy on every GPU it runs on, until the process
 * ends), and the call creates no stream, event or buffer.  Arguments as spb_forward, without the workspace; the
 * matching spb_backward_truncated then reads that array.  Differences from spb_forward:
 *   - a depth whose spb_workspace_size exceeds SPB_STATIC_WORKSPACE_BYTES is refused with SPB_ERR_WORKSPACE
 *     before anything is enqueued (the two perceptron workloads fit at every depth; the CNN and encoder
 *     workloads at full size do not);
 *   - the model's second stream is not created here, so unless an earlier spb_forward created it the backward
 *     pass stays on the caller's stream (same bits either way);
 *   - all models and all calls on one GPU share the one array, which keeps the last call's contents: a step
 *     (this call up to the end of its backward pass) must have completed on the device before the next
 *     spb_forward_static on that GPU is enqueued on another stream, or the two race.  Nothing needs to start at
 *     zero: every kernel writes what it later reads, pad columns included;
 *   - the first call on a device looks up the array's address and is best made outside a stream capture.
 * Errors: INVALID_ARG, DEPTH_RANGE, STATE, WORKSPACE (does not fit), HIP. */
#define SPB_STATIC_WORKSPACE_BYTES (8u << 20)
int spb_forward_static(spb_model* m, const void* x, const int32_t* labels, const int32_t* loss_rows,
                       int32_t stash_depth_k, float* loss_out, void* stream);

/* Backward pass over the top k units only (Sec. 2: a worker backpropagates a fixed suffix of the network
 * that starts at the output layer).  Requires a preceding spb_forward with
 * stash_depth_k >= k on the same workspace.  Overwrites (does not accumulate into) the gradient
 * buffers of units >= L-k and touches no other gradient buffer; the lowest visited unit gets its
 * parameter gradients but no input gradient is formed for it.  k = 0 enqueues nothing.
 * Errors: DEPTH_RANGE, STATE (no forward, deeper than stashed, gradient buffer of a visited unit
 * not bound), HIP. */
int spb_backward_truncated(spb_model* m, int32_t k, void* stream);

/* The gradients a worker sends after a depth-k step (Sec. 2: only the gradients it computed): one view per parameter of the top k units, output end first, and nothing for the
 * units below the cut.  out: host array of cap entries; n_out receives the count (0 for k = 0).
 * Errors: DEPTH_RANGE, INVALID_ARG (cap too small), STATE (gradients not bound). */
int spb_grad_buffers(const spb_model* m, int32_t k, spb_grad_view* out, int32_t cap, int32_t* n_out);

/* Read-only description of two tensors a step leaves in the caller's workspace, for tests and diagnosis that check
 * one unit at a time (Sec. 1: the gradient of a layer depends only on the layers after it, so a unit's backward
 * pass is fixed by the unit's input and the gradient entering it from above).  Host-only; nothing is enqueued.
 *   input        where a forward pass with stash depth k keeps the INPUT of unit `unit` (unit >= L - k)
 *   output_grad  where the gradient of the loss with respect to the unit's OUTPUT lies after
 *                spb_backward_truncated of depth exactly L - unit, i.e. with `unit` the lowest visited unit (a deeper
 *                backward pass reuses the buffer).  offset = SPB_VIEW_NONE for the top unit, which carries the loss.
 * A view is row-major [rows, cols] with `pitch` elements from row to row (NHWC tensors: rows = pixels, cols =
 * channels); offset is in bytes from the workspace base, or SPB_VIEW_CALLER_INPUT when the tensor is the x the
 * caller passed (unit 0), or SPB_VIEW_NONE.  relu_applied = 1 on a perceptron unit's output_grad: the mask of the
 * unit's own ReLU is already applied (it is the gradient at the unit's pre-activation).
 * Errors: DEPTH_RANGE, INVALID_ARG (unit below the cut of depth k). */
#define SPB_VIEW_CALLER_INPUT (-1)
#define SPB_VIEW_NONE (-2)
typedef struct spb_buffer_view {
  int64_t offset;
  int64_t rows, cols, pitch;
  int32_t dtype;         /* SPB_DTYPE_* */
  int32_t relu_applied;
} spb_buffer_view;
int spb_unit_io(const spb_model* m, int32_t stash_depth_k, int32_t unit, spb_buffer_view* input, spb_buffer_view* output_grad);

/* Fill with zeros the gradient buffers of the units below the cut, for callers that want dense
 * gradients.  Buffers bound as NULL are skipped. */
int spb_zero_absent_grads(spb_model* m, int32_t k, void* stream);

/* Depth of worker j (1-based) among n_workers (Sec. 2: the j-th worker backpropagates jL/k of the layers,
 * counted from the output; the paper does not say how the quotient is rounded: it is rounded up here, so
 * that the last worker always runs the full backward pass).  Host-only; *k receives ceil(j * L / n_workers).
 * Errors: INVALID_ARG (j outside 1..n_workers). */
int spb_worker_depth(const spb_model* m, int32_t j, int32_t n_workers, int32_t* k);

#define SPB_MAX_WORKERS 8

/* Parameter-server side of one iteration (Sec. 2): the partial gradients of n_workers workers, worker j having
 * backpropagated the top depths[j] units, are averaged per parameter over the workers that contributed to it
 * (c = number of workers with depths[j] >= L - unit), the learning rate of a parameter is lr * c / n_workers when
 * scale_lr is non-zero (Sec. 2 scales the rate with the number of contributors; the formula is this library's
 * reading) and lr otherwise, and the parameter takes one step of SGD with momentum and weight decay (Sec. 4.1):
 *     g = (1/c) * sum of the contributors' gradients;   v = momentum * v + g + weight_decay * w;   w = w - rate * v.
 * A parameter no worker contributed to (c = 0) is left untouched, and so is its velocity.
 *   depths        host array [n_workers], each in 0..L
 *   worker_grads  host array [n_workers * n_params] of device pointers, entry j * n_params + i = worker j's
 *                 float32 gradient of parameter i (dense, the parameter's shape); read only where worker j
 *                 contributes to parameter i, may be NULL elsewhere
 *   velocity      host array [n_params] of device pointers, float32, the parameter's shape, updated in place
 * The parameters are the buffers bound with spb_bind_params (model dtype; a bfloat16 parameter is rounded to
 * nearest-even after the float32 update) and are updated in place.  Enqueues on `stream`; allocates nothing.
 * Errors: INVALID_ARG (n_workers outside 1..SPB_MAX_WORKERS, null pointers where one is read), DEPTH_RANGE,
 * STATE (parameters not bound), HIP. */
int spb_aggregate_update(spb_model* m, int32_t n_workers, const int32_t* depths, void* const* worker_grads,
                         void* const* velocity, float lr, float momentum, float weight_decay, int32_t scale_lr,
                         void* stream);

/* Kernel timing.  When enabled, every kernel the model enqueues is bracketed by two HIP events on
 * the launch stream.  spb_read_kernel_timing waits for the recorded events, adds them up per kernel
 * class into out (host array of cap records; n_out receives the count) and clears the record.
 * Must not be enabled while the stream is being captured into a graph. */
int spb_set_kernel_timing(spb_model* m, int32_t enable);
int spb_read_kernel_timing(spb_model* m, spb_kernel_time* out, int32_t cap, int32_t* n_out);

/* Measurement aid: enqueue `count` back-to-back copies of the most recent matrix product of kernel class
 * `name` (as spb_read_kernel_timing reports it, e.g. "gemm_bf16_fwd 256x1024x1024") that ran while timing was enabled, on the same operands (the workspace of the
 * last step must still be alive; the copies rewrite that product's output with the same values).  Two events
 * around the call give the kernel's duration without the per-launch event overhead.
 * Errors: INVALID_ARG, STATE (no such product recorded), HIP. */
int spb_replay_kernel(spb_model* m, const char* name, int32_t count, void* stream);

/* ---- Placement of training tasks on devices and in time (Sec. 3, "Scheduling Algorithm") -------------------
 * Host code only: no GPU is touched and every pointer below is a HOST pointer.
 *
 * A job is a chain of iterations; an iteration is one task per worker; the tasks of iteration i + 1 become
 * ready when every task of iteration i of the same job has ended.  Under SPB the workers of a job differ in
 * run time and memory, so tasks are placed one by one: ready tasks wait in a priority queue keyed by
 * resource * duration (largest first; ties to the smaller job, iteration, worker), and the task taken from it
 * goes to the device on which it can start earliest.  A device runs one task at a time and a task may fill a gap
 * left between tasks placed before it.  On the device that ran the same worker in the previous iteration a task
 * is ready when that iteration has ended; on any other device (and for a job's first iteration, on every device)
 * gamma * model_size later, the time it takes to bring the model there.  Between devices that offer the same
 * start the previous device wins, then the lowest index.
 * gang != 0 gives the baseline the section compares with: the workers of an iteration start together, on as many
 * devices, at the earliest time at which that many are free for the slowest worker's duration, and hold them
 * that long; a worker keeps its previous device when that one is free then, the others take the free devices of
 * lowest index and need the start-up delay; iterations are ordered by (sum of resources) * (slowest duration).
 * (The paper normalises resource and duration by cluster constants, which does not change the order; what it
 * leaves open - the tie rules, exclusive devices, the first iteration's delay - is as stated here.) */
typedef struct spb_sched_job {
  double arrival;           /* earliest start of the job's first iteration, >= 0 */
  double model_size;        /* in the unit gamma is per, >= 0 */
  int32_t iterations;       /* >= 0 */
  int32_t workers;          /* >= 1 */
  const double* durations;  /* [workers] run time of each worker's task, > 0 */
  const double* resources;  /* [workers] GPU resource (e.g. peak memory) of each worker's task, in [0, capacity] */
} spb_sched_job;

typedef struct spb_sched_task {
  int32_t job, iteration, worker;
  int32_t machine;    /* device index in [0, n_machines) */
  int32_t moved;      /* 1 when the previous iteration of this worker ran on another device */
  double start, end;  /* the task computes during [start, end) */
  double held_until;  /* its device is taken during [start, held_until): end, or the gang's end */
} spb_sched_task;

/* Places every task of every job.  out receives the tasks in the order in which they were placed (cap entries;
 * n_out receives the number of tasks, also when cap is too small), makespan the latest held_until (0 without
 * tasks).  Errors: INVALID_ARG (null pointer, a value outside the ranges above, n_machines < 1, a gang wider
 * than the cluster, cap too small). */
int spb_schedule_tasks(const spb_sched_job* jobs, int32_t n_jobs, int32_t n_machines, double gamma, double capacity,
                       int32_t gang, spb_sched_task* out, int64_t cap, int64_t* n_out, double* makespan);

#ifdef __cplusplus
}
#endif
#endif /* SPB_H */
