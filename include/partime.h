/*
 * partime.h - C ABI of the MI355X pipelined online learner.
 *
 * The library runs, on ONE GPU, the per-tick hot path of pipelined online
 * learning over a data stream (Sec. III and Algorithm 1 of the PARTIME paper):
 * at every stream tick each stage h of a feed-forward network
 *   - runs forward on what stage h-1 produced one tick earlier (Eq. 6),
 *   - takes the error stage h+1 produced one tick earlier (Eq. 11),
 *   - forms its weight gradient at this tick's input and weights (Eq. 9),
 *   - publishes its own input-error, computed with the not yet updated weights,
 *   - and applies its SGD update at once (Algorithm 1, last two steps).
 * All stages of a tick run concurrently in one grouped kernel launch.
 *
 * Conventions
 *   - Every function returns PT_OK (0) or a negative PT_E* code; on failure
 *     partime_last_error() gives a thread-local description.  Nothing throws.
 *   - Pointers named *_host are host memory, *_dev are device memory on the
 *     current HIP device.  The library never takes ownership of caller memory.
 *   - partime_step / partime_infer only enqueue work on the stream given in the
 *     configuration and never synchronise the host; caller buffers must stay
 *     alive until that stream has passed the call.
 *   - Vectors are fp32.  Weights are row-major [out][in] fp32 on the host side
 *     of every call, whatever the device storage type.
 */
#ifndef PARTIME_H
#define PARTIME_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct partime_ctx partime_ctx; /* opaque; owns weights, biases, ping-pong buffers */

/* layer kind */
enum { PT_DENSE = 0, PT_CONV3X3 = 1, PT_GAP_DENSE = 2 };
/* activation: identity, ReLU (derivative 0 at 0), GELU (exact erf form) */
enum { PT_ID = 0, PT_RELU = 1, PT_GELU = 2 };
/* loss at the last stage: MSE = mean_i (o_i - y_i)^2 ; CE = -log softmax(o)[y] ; mean over streams */
enum { PT_LOSS_NONE = 0, PT_LOSS_MSE = 1, PT_LOSS_CE = 2 };
/* device storage of the weights; all arithmetic is fp32; bf16 stores round to nearest even */
enum { PT_F32 = 0, PT_BF16 = 1 };
/* how a block of ticks is executed */
enum { PT_EXEC_AUTO = 0, PT_EXEC_LAUNCH_PER_TICK = 1, PT_EXEC_PERSISTENT = 2 };
/* update rule: plain SGD (Algorithm 1), or Adam with bias correction (used in Sec. V-D), one optimiser step per tick */
enum { PT_OPT_SGD = 0, PT_OPT_ADAM = 1 };
/* error codes */
enum { PT_OK = 0, PT_EINVAL = -1, PT_ESHAPE = -2, PT_ENOMEM = -3, PT_EHIP = -4, PT_EUNSUPPORTED = -5 };

typedef struct {
  int kind;            /* PT_DENSE: in_dim -> out_dim.  PT_CONV3X3: c_in x h x w -> c_out x h x w,
                          stride 1, pad 1.  PT_GAP_DENSE: mean over h x w of c_in planes, then c_in -> out_dim */
  int act;             /* PT_ID / PT_RELU / PT_GELU */
  int in_dim, out_dim; /* dense sizes */
  int c_in, c_out, h, w;
  int skip_from;       /* -1, or the index of an earlier layer whose output (same size) is added to this layer's
                          output after the activation (skip connections of Sec. V-C; the tensor and its gradient
                          cross the stages in between one per tick, like the main path).  Dense layers (any stream
                          count offered) and conv layers (equal channel counts); not PT_EXEC_PERSISTENT; one skip
                          per source layer; not into the last layer. */
} pt_layer;

typedef struct {
  int n_layers;
  const pt_layer *layers; /* host; copied */
  int depth;              /* D, number of pipeline stages (Eq. 3) */
  const int *balance;     /* host, depth entries: layers per stage (Eq. 3), sum = n_layers; NULL = one layer per stage.
                             Inside a stage back-propagation is exact (Eq. 5); only stage boundaries carry the delay.
                             Several layers per stage: not PT_EXEC_PERSISTENT; dense layers (any stream count offered), or conv
                             layers (one stream) with the pooled dense layer as a stage of its own. */
  int n_streams;          /* S independent streams sharing the weights; gradients and loss are means over S.
                             1, 32, or a multiple of 64 up to 1024 (the last: the slots of a replay batch, Sec. V-D);
                             S > 1 takes dense layers and bf16 weights and rounds what
                             enters a product to bf16 */
  int w_dtype;            /* PT_F32 / PT_BF16 */
  int loss;               /* PT_LOSS_* */
  float lr;               /* SGD step size */
  int target_delay;       /* k >= 0: the last stage at tick t is scored against the target supplied at tick t-k.
                             k = 0 is the literal pairing of the text under Eq. 10; k = depth-1 pairs every
                             output with the target of the sample it was computed from (Eq. 7). */
  int exec_mode;          /* PT_EXEC_* */
  void *hip_stream;       /* hipStream_t on which all work is enqueued (NULL = the null stream) */
  int optimizer;          /* PT_OPT_*.  Adam: every kind of pipeline, not PT_EXEC_PERSISTENT; moments fp32, start at 0 */
  float beta1, beta2, eps; /* Adam only: m <- beta1 m + (1-beta1) g, v <- beta2 v + (1-beta2) g^2,
                              w <- w - lr (m / (1-beta1^n)) / (sqrt(v / (1-beta2^n)) + eps), n = tick + 1 */
} partime_config;

/*
 * Build a pipeline.  w_host[i] / b_host[i] are the fp32 initial weights and
 * biases of layer i (row-major [out][in]; conv [c_out][c_in][3][3]); they are
 * copied (and rounded to bf16 if so configured).  All buffers start at zero
 * and the tick counter at 0.  The loss gradient is held at zero for ticks
 * < max(depth-1, target_delay): until then no real sample/target pair exists
 * at the last stage.  *out receives the context.
 * Errors: PT_EINVAL (null pointers, bad enum, sizes <= 0), PT_ESHAPE (layer i+1
 * input does not match layer i output, balance does not sum to n_layers),
 * PT_EUNSUPPORTED (a configuration no kernel covers yet), PT_ENOMEM, PT_EHIP.
 */
int partime_init(const partime_config *cfg, const float *const *w_host, const float *const *b_host,
                 partime_ctx **out);

/*
 * n_ticks learning ticks (Algorithm 1: forward, backward, update, for all stages).
 *   x_dev      [n_ticks][S][in]   fp32 stream samples, one per tick
 *   target_dev [n_ticks][S][out] fp32 (MSE) or [n_ticks][S] int32 class ids (CE)
 *   out_dev    [n_ticks][S][out]  row t = output of the last stage at that tick, i.e. the
 *                                 prediction for the sample that entered depth-1 ticks earlier (Eq. 7);
 *                                 rows of the first depth-1 ticks of a fresh pipeline are written but meaningless
 *   loss_dev   [n_ticks]          loss at each tick (0 while the loss gradient is held at zero); may be NULL
 * n_ticks = 0 is a no-op.  Errors: PT_EINVAL (null ctx / pointers, n_ticks < 0), PT_EHIP.
 */
int partime_step(partime_ctx *ctx, const float *x_dev, const void *target_dev, int n_ticks, float *out_dev,
                 float *loss_dev);

/*
 * partime_step for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical results; the loss partials that
 * partime_step keeps in a buffer of the context (one float per tile of the last stage and tick, summed in a fixed
 * order by a small kernel at the end of each block of 1024 ticks) live in a static device array of the library
 * instead (1 MiB + 4 KiB per GPU, held from the first partime_init on that GPU until the process ends), whose
 * address is looked up once per device.  The call itself allocates and frees nothing, on the host or the device.
 * Limits: dense pipelines of one stream run with one launch per tick (any `balance`, SGD or Adam, skip connections);
 * at most 256 tiles in the last stage.  Anything else: PT_EUNSUPPORTED, nothing is enqueued.
 * Every call on a GPU shares that GPU's array, whatever the context or stream: calls that overlap in time on one GPU
 * race on it (the losses of the overlapping calls are then undefined; weights and outputs are not affected).  Nothing
 * in it has to start at zero: every slot a call reads it has written before, so the leftovers of an earlier, larger
 * call are never seen.
 */
int partime_step_noalloc(partime_ctx *ctx, const float *x_dev, const void *target_dev, int n_ticks, float *out_dev,
                         float *loss_dev);

/* n_ticks forward-only ticks (Eq. 6 only) on the same buffers; weights are left untouched. */
int partime_infer(partime_ctx *ctx, const float *x_dev, int n_ticks, float *out_dev);

/* Synchronous copy-out / copy-in of layer i's weights and biases as fp32 (either pointer may be NULL). */
int partime_get_state(partime_ctx *ctx, int layer, float *w_host, float *b_host);
int partime_set_state(partime_ctx *ctx, int layer, const float *w_host, const float *b_host);

/*
 * Synchronous access to the inter-stage buffers, for checkpoints and single-tick checks.
 *   which = 0: what stage `stage` published for stage+1 (activation, [S][stage out size])
 *   which = 1: the input-error stage `stage` published for stage-1 ([S][stage in size])
 *   which = 2: the targets of the last target_delay ticks, oldest first, that the coming ticks will be scored
 *              against (text under Eq. 10 with the pairing of Eq. 7): target_delay x one tick's targets, copied as
 *              the 4-byte elements they were supplied in (fp32, or int32 class ids behind the float pointer);
 *              stage and half are ignored; nothing is copied when target_delay = 0
 *   which = 3 / 4: the delay lines of the skip connection that ends in layer `stage` (a layer index here): 3 = the
 *              skipped tensor on its way forward, 4 = the gradient on its way back, each [S][layer out size]
 *              (conv: [C][H][W]); `half` is the AGE of the entry in ticks, 0 = written during the last tick ...
 *              d - 1 = the one the coming tick consumes (d = stage boundaries the skip crosses; a skip inside a stage
 *              has nothing in flight between ticks).  Ages count back from the tick counter: use after
 *              partime_set_tick, and not across inference ticks (those move the tensors, not the gradients).
 *   half  = 0/1 (which < 2): the half written at even / odd ticks.
 * Pipelines of 64 and more streams keep activations rounded to bf16: those come back, and are taken, as such.
 */
int partime_get_buffer(partime_ctx *ctx, int which, int stage, int half, float *host);
int partime_set_buffer(partime_ctx *ctx, int which, int stage, int half, const float *host);

int partime_get_tick(partime_ctx *ctx, int64_t *tick);
int partime_set_tick(partime_ctx *ctx, int64_t tick);
int partime_set_lr(partime_ctx *ctx, float lr);

/*
 * Wait until the stream has passed everything this context enqueued and report deferred device-side
 * failures: in PT_EXEC_PERSISTENT mode the ticks of a call run inside one kernel and are separated by a
 * grid-wide barrier whose wait is bounded; if it ever runs out the kernel stops and PT_EHIP is returned
 * here (and by partime_get_state / partime_get_buffer).
 */
int partime_sync(partime_ctx *ctx);

/* Zero every inter-stage buffer and the target history, tick = 0; weights are kept. */
int partime_reset(partime_ctx *ctx);

void partime_destroy(partime_ctx *ctx);

/* Thread-local description of the last failure on this thread ("" if none). */
const char *partime_last_error(void);

/* Synchronous copy-out / copy-in of layer i's Adam moments (first, second; weights in the layout of partime_get_state, biases);
 * any pointer may be NULL.  PT_EINVAL if the pipeline runs plain SGD. */
int partime_get_opt_state(partime_ctx *ctx, int layer, float *m_w_host, float *v_w_host, float *m_b_host, float *v_b_host);
int partime_set_opt_state(partime_ctx *ctx, int layer, const float *m_w_host, const float *v_w_host,
                          const float *m_b_host, const float *v_b_host);

/* Number of kernel launches the last partime_step / partime_infer call enqueued (diagnostic). */
int partime_last_launch_count(partime_ctx *ctx);

/*
 * Measured streaming ceiling of the current device, to put beside the published HBM peak when the
 * weight-streaming kernels (forward + update of Algorithm 1: every weight read and rewritten per tick) are
 * judged: runs a kernel with no arithmetic over a private buffer of `bytes` bytes `iters` times on the null
 * stream, for three grid sizes, and returns the best GB/s in *gbps_out.  mode 0 = read only, 1 = write only, 2 = in-place read + write (bytes
 * counted twice).  Synchronises the host; allocates and frees its buffer.  Errors: PT_EINVAL, PT_EHIP.
 */
int partime_bandwidth_probe(size_t bytes, int mode, int iters, double *gbps_out);

#ifdef __cplusplus
}
#endif
#endif /* PARTIME_H */
