/*
 * aet_sgd.h -- C ABI of the MI355X (gfx950) implementation of the AET-SGD hot path:
 * many client model replicas resident on one GPU, each running local SGD rounds whose
 * length follows the linearly increasing sample-size threshold, accumulating the round's
 * gradient sum U; a server step that applies the received U's under a deterministic
 * delay schedule and rebroadcasts the global model.
 *
 * Paper: arXiv 2112.13935.  Citations below name its sections, equations and algorithms
 * ("Algorithm 1" = Initial Setup of AET-SGD, "Algorithm 2" = AET-SGD Framework with the
 * procedures Receive, Synchronize and MainComputeNode).
 *
 * Conventions
 *   - All floating point is fp32 on the device.
 *   - "DEVICE" pointers are HIP device memory owned by the caller (allocate them with
 *     PyTorch or hipMalloc) and must stay valid until aet_destroy.  "HOST" pointers are
 *     ordinary host memory, read or written during the call only.
 *   - The library allocates no device memory: everything it needs lives in the
 *     workspace the caller passes to aet_init (size from aet_workspace_bytes).
 *   - Every call returns an aet_status; on anything but AET_OK nothing has been applied
 *     and aet_last_error() describes the problem.  Nothing aborts or throws across the
 *     boundary.
 *   - Work is enqueued on the HIP stream given to aet_init and is asynchronous; calls
 *     that return data to HOST memory synchronise that stream.
 *   - A context is not thread safe; use one host thread per context.
 *
 * Canonical parameter layout (w0, aet_get_weights, aet_get_U): layers in order, for each
 * layer its weights then its bias; dense weights W[out][in] row-major; convolution
 * weights W[cout][cin][kh][kw]; a convolution/pool output is flattened in C,H,W order
 * before a dense layer.  Samples are rows of in_c*in_h*in_w floats in C,H,W order.
 */
#ifndef AET_SGD_H
#define AET_SGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct aet_ctx aet_ctx; /* opaque, owned by the library */

typedef enum {
    AET_OK = 0,
    AET_EINVAL = -1, /* bad argument, unsupported model, round length not a multiple of batch */
    AET_ENOMEM = -2, /* workspace too small, host allocation failed, no free U slot */
    AET_EHIP = -3,   /* a HIP call or kernel launch failed */
    AET_ESTATE = -4  /* call not valid in this state (e.g. no such message in flight) */
} aet_status;

#define AET_MAX_LAYERS 16
#define AET_CONV 0  /* k x k convolution, stride 1, zero padding `pad`, optional ReLU */
#define AET_POOL 1  /* 2 x 2 max pooling, stride 2 (input height and width must be even) */
#define AET_DENSE 2 /* fully connected, optional ReLU */

typedef struct {
    int32_t type; /* AET_CONV / AET_POOL / AET_DENSE */
    int32_t cout; /* output channels (conv) or features (dense); ignored for pool */
    int32_t k;    /* kernel size (conv: 1, 2, 3 or 5) */
    int32_t pad;  /* zero padding on each side (conv) */
    int32_t relu; /* 1: ReLU after the affine map */
} aet_layer;

/* The loss f(w; xi) of eq. (3): softmax cross-entropy of the last (dense, no ReLU)
 * layer's outputs against the label.  `batch` samples are averaged per SGD recursion. */
typedef struct {
    int32_t in_c, in_h, in_w; /* one sample = in_c*in_h*in_w floats */
    int32_t n_layers;         /* 1 .. AET_MAX_LAYERS */
    int32_t batch;            /* mini-batch size B >= 1 */
    aet_layer layers[AET_MAX_LAYERS];
} aet_model_desc;

/* A client's local data set D_c (Algorithm 2, MainComputeNode input). */
typedef struct {
    const float *X;    /* DEVICE, n_samples rows */
    const int32_t *y;  /* DEVICE, n_samples labels in [0, classes) */
    int64_t n_samples; /* 1 .. 2^31-1 */
} aet_shard;

/* Linearly increasing sample-size threshold (Section 3.1; Table 5: s_i = a*i^p + b with
 * p = 1): local round i of a client ends after s_i = a*i + b samples, i.e. s_i / batch
 * recursions; s_i must be a multiple of batch (s_i = 0 is legal: an empty round whose
 * message carries U = 0).  Every client performs `rounds` local rounds, i = 0..rounds-1. */
typedef struct {
    int64_t a, b;
    int32_t rounds;
} aet_threshold;

/* Round step size (Experiments, "Objective function"; Section 3.1): constant within a
 * round, eta_i = eta0 / (1 + beta * t^power), t = recursions this client has completed
 * before the round.  The paper uses power = 1/2; beta = 0 gives a constant step.
 * Evaluated in double precision and rounded once to fp32. */
typedef struct {
    double eta0, beta, power;
} aet_eta;

/* Deterministic stand-in for the paper's injected random computation and network delays
 * (Section "System delay"; Experiments, "System delay"), in units of ticks (one tick =
 * one aet_run_round + aet_server_aggregate pair):
 *   compute_factor[c] >= 1 : a local round of client c occupies that many ticks;
 *   is_straggler[c] != 0   : each message of c spends delay_min..delay_max extra ticks in
 *                            the network, drawn by a counter hash of (seed, c, round);
 *   d_max >= 0             : the delay checkpoint of Algorithm 2 (Synchronize): client c
 *                            does not start round i while max over the other clients e of
 *                            (i - H_e) exceeds d_max, H_e = messages of e applied so far;
 *                            d_max < 0 switches the checkpoint off. */
typedef struct {
    const int32_t *compute_factor; /* HOST, n_clients entries, or NULL = all 1 */
    const uint8_t *is_straggler;   /* HOST, n_clients entries, or NULL = none */
    int32_t delay_min, delay_max;  /* 0 <= delay_min <= delay_max < max_inflight */
    uint64_t seed;
    int32_t d_max;
} aet_delay;

/* Number of parameters P of the model, or -1 if the description is not supported. */
int64_t aet_n_params(const aet_model_desc *model);

/* Bytes of DEVICE workspace aet_init needs (0 if the arguments are invalid).
 *   max_inflight : U messages one client may have posted and not yet applied
 *                  (delay_max + 1 is always enough);
 *   max_rounds   : upper bound on local rounds per client (sizes the loss log). */
size_t aet_workspace_bytes(const aet_model_desc *model, int32_t n_clients, int32_t max_inflight,
                           int32_t max_rounds);

/* Setup (Algorithm 1, first line; Algorithm 2, MainComputeNode initialisation): the
 * global model and every client's local model start as w0; local round counters,
 * recursion counters and the receive history H are zero; time starts at tick 0.
 *   shards        HOST array of n_clients records (the records hold DEVICE pointers)
 *   w0            HOST, P floats, canonical layout
 *   seed          seed of the per-client sample-index streams
 *   workspace     DEVICE, 256-byte aligned, workspace_bytes >= aet_workspace_bytes(...)
 *   hip_stream    a hipStream_t passed as void* (NULL = the default stream)
 * Sample q (counting from 0 over the client's whole life) of client c is row
 *   ((h >> 32) * n_samples) >> 32,  h = SplitMix64 stream value number q of the stream
 * keyed by (seed, client): uniform with replacement (the sampling step of Algorithm 2,
 * MainComputeNode), a pure function of (seed, c, q). */
aet_status aet_init(aet_ctx **out, const aet_model_desc *model, int32_t n_clients,
                    const aet_shard *shards, const float *w0, uint64_t seed, void *workspace,
                    size_t workspace_bytes, int32_t max_inflight, int32_t max_rounds,
                    void *hip_stream);

/* aet_init for callers that cannot allocate device or pinned host memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the context's
 * workspace is an array inside the library, AET_STATIC_WORKSPACE_BYTES per GPU, held from
 * the moment the library is loaded until the process ends.  This call and every later call
 * on such a context allocate nothing with HIP: no hipMalloc / hipHostMalloc / hipFree, no
 * events; the round and arrival records reach the device in kernel arguments instead of
 * through pinned staging buffers.
 *   w0_dev   DEVICE, P floats, canonical layout (read before the call returns)
 *   the other arguments as for aet_init; the context lives on the current device.
 * AET_ENOMEM (with the two sizes in aet_last_error(NULL)) when
 * aet_workspace_bytes(model, n_clients, max_inflight, max_rounds) exceeds
 * AET_STATIC_WORKSPACE_BYTES.  Every such context on one GPU uses the same array, which
 * keeps what the last one left (the part the new context uses is cleared by this call):
 * only ONE may be alive per GPU at a time -- a second aet_init_static on that GPU before
 * aet_destroy of the first returns AET_ESTATE -- and work of a destroyed context that is
 * still running on another stream would race with the new one (aet_destroy synchronises
 * the context's own stream).  Contexts made by aet_init are not affected. */
#define AET_STATIC_WORKSPACE_BYTES (64 * 1024 * 1024)
aet_status aet_init_static(aet_ctx **out, const aet_model_desc *model, int32_t n_clients,
                           const aet_shard *shards, const float *w0_dev, uint64_t seed,
                           int32_t max_inflight, int32_t max_rounds, void *hip_stream);

/* One tick of local rounds (Algorithm 2, MainComputeNode: one pass of the round loop for
 * every client that is idle, has rounds left and passes the delay checkpoint).  Such a
 * client c, at its round i:
 *   adopts the server's current global model (client-server paragraph of the
 *   Introduction: the server broadcasts its most recent model), or, once a topology is
 *   set, goes on from its own model (Algorithm 2 as printed);
 *   h = 0, U = 0; for each of the s_i / batch recursions: draws `batch` sample indices,
 *   g = mean of grad f(w_c; xi) over them, w_c <- w_c - eta_i g, U <- U + g;
 *   posts the message (c, U_i, i) with arrival tick
 *   now + compute_factor[c] - 1 + network delay, and is busy for compute_factor[c] ticks.
 * All clients of the tick run inside the same kernel launches.
 *   n_finished, finished_client, finished_round : HOST outputs (capacity n_clients; any
 *   may be NULL): the clients that ran a round this tick, ascending, and their round i. */
aet_status aet_run_round(aet_ctx *ctx, const aet_threshold *thr, const aet_eta *eta,
                         const aet_delay *delay, int32_t *n_finished, int32_t *finished_client,
                         int32_t *finished_round);

/* Server form of Receive (Algorithm 2): every message (v, U, k) whose arrival tick is the
 * current tick is applied as  w_global <- w_global - agg_scale * eta_k * U  with the
 * SENDER's round step size eta_k, H_v <- H_v + 1; arrivals of one tick are taken in
 * (k ascending, v ascending) order.  Then the tick counter advances.  agg_scale = 1 is
 * the paper's rule; 1/n_clients averages the clients' displacements.
 *   n_applied, applied_client, applied_round : HOST outputs (capacity: the number of
 *   messages in flight, at most n_clients * max_inflight; any may be NULL). */
aet_status aet_server_aggregate(aet_ctx *ctx, float agg_scale, int32_t *n_applied,
                                int32_t *applied_client, int32_t *applied_round);

/* Setup (Algorithm 1): round lengths from coin flips.  After this call the threshold given
 * to aet_run_round is the GLOBAL sequence s_i = a*i + b (samples over all nodes), each of
 * the s_i / batch recursions of global round i is assigned to node c with probability
 * p_c = weights[c] / sum(weights), and node c's round i has
 *   s_{i,c} = batch * |{ t : a(i,t) = c }|     (E[s_{i,c}] = p_c s_i; 0 is possible: the
 * node then sends an empty message).  a(i,t): value t of the SplitMix64 stream keyed by
 * (seed, round i), top 32 bits mapped onto [0, sum(weights)) by multiply-shift, located
 * in the cumulative weights; integer arithmetic only, a pure function of (seed, i, t).
 *   weights  HOST, n_clients entries, sum in [1, 2^32); copied during the call.
 * Only before the first round (AET_ESTATE later). */
aet_status aet_set_setup(aet_ctx *ctx, const uint32_t *weights, uint64_t seed);

/* Peer-to-peer form (Algorithm 2 as printed; Section 2.2.1: undirected topology, the
 * neighbour list of every node is given).  After this call every node keeps its own model
 * from round to round, a message goes to the sender's neighbours (aet_receive), and the
 * delay checkpoint of node c looks at its neighbours only:  max over e in N(c) of
 * (i_c - H_e) > d_max  holds c back.  Only before the first round.
 *   nbr_off   HOST, n_clients + 1 entries, nbr_off[0] = 0, not decreasing
 *   nbr       HOST, nbr_off[n_clients] entries: the neighbours of c are
 *             nbr[nbr_off[c] .. nbr_off[c+1]), strictly ascending, never c itself, and v is
 *             listed for c exactly when c is listed for v (else AET_EINVAL)
 *   workspace DEVICE, 256-byte aligned, at least aet_topology_workspace_bytes(n_clients,
 *             nbr_off[n_clients]) bytes; owned by the caller, kept alive until aet_destroy.
 * The host arrays are copied during the call. */
size_t aet_topology_workspace_bytes(int32_t n_clients, int32_t n_neighbour_entries);
aet_status aet_set_topology(aet_ctx *ctx, const int32_t *nbr_off, const int32_t *nbr, void *workspace,
                            size_t workspace_bytes);

/* Receive as Algorithm 2 prints it, for a context with a topology: every message (v, U, k)
 * whose arrival tick is the current tick is applied by each neighbour r of v to its own
 * model,  w_r <- w_r - scale * eta_k * U  (sender's round step size; scale = 1 is the
 * paper's rule), H_v <- H_v + 1.  A node applies the tick's arrivals in (k ascending, v
 * ascending) order.  A node whose round occupies several ticks did its recursions in the
 * round's first tick, so what arrives meanwhile lands on the model as that round left it.
 * Then the tick counter advances.
 *   n_applied, applied_sender, applied_round : HOST outputs, the messages delivered
 *   (capacity: the number of messages in flight, at most n_clients * max_inflight; any may
 *   be NULL).
 * AET_ESTATE without a topology; aet_server_aggregate returns AET_ESTATE with one. */
aet_status aet_receive(aet_ctx *ctx, float scale, int32_t *n_applied, int32_t *applied_sender,
                       int32_t *applied_round);

/* Driver loop: repeats { aet_run_round; aet_server_aggregate } (with a topology:
 * { aet_run_round; aet_receive }, agg_scale being the scale) with the same parameters
 * until every client has completed thr->rounds local rounds and the message queue has
 * drained, or max_ticks ticks have run.  *ticks_done (HOST, may be NULL) receives the
 * number of ticks run; it is valid also when a tick fails. */
aet_status aet_run_ticks(aet_ctx *ctx, const aet_threshold *thr, const aet_eta *eta,
                         const aet_delay *delay, float agg_scale, int32_t max_ticks,
                         int32_t *ticks_done);

/* U of the message (client, round) while it is in flight (posted, not yet applied).
 * dst: P floats, HOST if on_host != 0 (synchronises), else DEVICE (enqueued). */
aet_status aet_get_U(aet_ctx *ctx, int32_t client, int32_t round, float *dst, int32_t on_host);

/* client < 0: the global model; else the local model w_c as its last round left it. */
aet_status aet_get_weights(aet_ctx *ctx, int32_t client, float *dst, int32_t on_host);

/* Import: overwrite the global model (client < 0) or the local model w_c with P floats in
 * the canonical layout.  src: HOST if on_host != 0 (copied before the call returns), else
 * DEVICE (enqueued on the stream).  Counters, queue and history are left as they are. */
aet_status aet_set_weights(aet_ctx *ctx, int32_t client, const float *src, int32_t on_host);

/* Bookkeeping of local round `round` of `client` (HOST outputs):
 *   ints[6] = { s_i, recursions m_i, first sample counter q0, recursions before the round
 *               t0, start tick, arrival tick };
 *   dbls[2] = { eta_i (the fp32 value used), mean training loss over the round's
 *               recursions }.  Synchronises the stream. */
aet_status aet_get_round_info(aet_ctx *ctx, int32_t client, int32_t round, int64_t *ints,
                              double *dbls);

/* The sample indices client `client` draws for sample counters q0 .. q0+count-1, computed
 * by the device code path that the round kernels use.  dst: HOST, count entries,
 * count <= 65536.  Synchronises. */
aet_status aet_debug_sample_indices(aet_ctx *ctx, int32_t client, int64_t q0, int32_t count,
                                    int32_t *dst);

/* 1 when every client has completed `rounds` local rounds and no message is in flight. */
int32_t aet_all_done(const aet_ctx *ctx, int32_t rounds);
int64_t aet_tick(const aet_ctx *ctx);
/* messages applied so far from `client` (the history H of Algorithm 2) */
int64_t aet_history(const aet_ctx *ctx, int32_t client);
/* number of messages in flight */
int64_t aet_inflight(const aet_ctx *ctx);

/* Block until everything enqueued so far has finished. */
aet_status aet_synchronize(aet_ctx *ctx);

/* Restart the run without re-creating the context: the global model goes back to the w0
 * given to aet_init (a replica is refreshed when its next round adopts the global
 * model); round counters, recursion and sample counters, the history H, the message
 * queue and the tick counter are cleared.  Enqueued, no sync. */
aet_status aet_reset(aet_ctx *ctx);

/* Which engine runs the local rounds, and what it needs from the device.
 *   - softmax regression (one dense layer, batch 1, 10 classes, up to 3072 inputs): one
 *     workgroup per client runs the whole round with the replica in registers;
 *   - dense-ReLU-dense models (batch 16 or 32, hidden width a multiple of 16 up to 256, up
 *     to 896 inputs): a CLUSTER of workgroups per client runs the whole round and
 *     exchanges partial sums through tagged records in the workspace.  PRECONDITION: all
 *     workgroups of a cluster must be resident on the GPU together.  The launcher sizes its
 *     launches from the occupancy the device reports for an otherwise idle GPU; if other
 *     work occupies compute units at the same time (another stream, process or a
 *     compute-unit mask) a cluster may not become resident.  The wait of a workgroup for
 *     its peers is bounded: when it expires the kernel raises an error flag and still runs
 *     to its end (nothing hangs), the results of that launch are invalid, and the next call
 *     that synchronises (aet_synchronize, any getter with on_host != 0, aet_get_round_info)
 *     returns AET_EHIP; from then on every call on the context returns AET_ESTATE.  There
 *     is no fall-back to another engine inside a context: create a new one (after
 *     aet_test_select_kernels(1, 0) it runs on the layer-by-layer engine);
 *   - every other model: one short kernel sequence per recursion (layer-by-layer engine).
 *
 * Test hook: contexts created after this call use the layer-by-layer engine for every
 * model (force_layer_engine != 0) and / or its plain-FMA kernels instead of the matrix-core
 * ones (plain_layers != 0), so that the kernel sets can be checked against each other and
 * against the oracle.  Process-wide; (0, 0) restores the defaults.  It also changes what
 * aet_workspace_bytes returns. */
void aet_test_select_kernels(int32_t force_layer_engine, int32_t plain_layers);

/* Optional kernel timing for measurement harnesses.  The library's kernels are grouped
 * in families (aet_profile_family_name gives each family's kernel name); while a family
 * is enabled, every launch of it is bracketed by a pair of HIP events recorded on the
 * context's stream.  aet_profile_read synchronises, then returns the number of launches
 * and the sum of their durations in milliseconds since the last reset.
 * family = -1 in aet_profile_enable means all families. */
int32_t aet_profile_families(void);
const char *aet_profile_family_name(int32_t family);
aet_status aet_profile_enable(aet_ctx *ctx, int32_t family, int32_t on);
aet_status aet_profile_read(aet_ctx *ctx, int32_t family, int64_t *launches, double *total_ms,
                            int32_t reset);

/* Text of the last error of this context (ctx == NULL: of the last failed aet_init). */
const char *aet_last_error(const aet_ctx *ctx);

/* Release host resources.  The workspace and the shards are the caller's. */
void aet_destroy(aet_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* AET_SGD_H */
