// C ABI and host scheduler of the AET-SGD library: per-client round counters, the
// threshold s_i = a*i + b, the round step size, sample counters, the message queue with
// its deterministic delays, and the order in which arrivals are aggregated.  All of it
// is integer bookkeeping on the host; the floating-point work is enqueued as kernels.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/aet_sgd.h"
#include "aet_device.h"
#include "aet_internal.h"

using namespace aet;

// ---- workspace inside the library, for aet_init_static ---------------------------------
// One array per GPU (every device that loads the code object holds its own copy at its own
// address).  Host code never uses the array's name as an address: the device address is
// looked up once per device (scratch_address) and that pointer is what kernels, copies and
// clears get.
static constexpr size_t kStaticBytes = (size_t)AET_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticBytes];
static constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices] = {};
static const aet_ctx *g_scratch_owner[kMaxDevices] = {};

static hipError_t scratch_address(int dev, void **ptr) {
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

// Records that a context without pinned staging buffers hands to the device: they travel
// in the kernel arguments and one small kernel drops them where the round / server kernels
// read them (stream-ordered, so nothing has to be fenced).
constexpr int kPutParams = 48;
struct ParamsPut { RoundParams p[kPutParams]; };
__global__ void k_put_params(const ParamsPut pack, int count, RoundParams *__restrict__ dst) {
    if ((int)threadIdx.x < count) dst[threadIdx.x] = pack.p[threadIdx.x];
}
constexpr int kPutArrivals = 224;
struct ArrivalsPut { Arrival a[kPutArrivals]; };
__global__ void k_put_arrivals(const ArrivalsPut pack, int count, Arrival *__restrict__ dst) {
    if ((int)threadIdx.x < count) dst[threadIdx.x] = pack.a[threadIdx.x];
}
__global__ void k_clear_bytes16(uint4 *__restrict__ p, size_t n16) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n16) p[i] = uint4{0u, 0u, 0u, 0u};
}

namespace {

constexpr int kRing = 4;            // pinned staging buffers in flight
constexpr int kDebugIdx = 65536;    // capacity of the debug index buffer
constexpr uint64_t kTagSample = 0;  // stream purposes of the counter hash
constexpr uint64_t kTagNet = 1;
constexpr uint64_t kTagSetup = 2;

struct Msg {
    int32_t c, k;
    float eta;
    int64_t arrival;
    int slot;
};

struct RoundRec {
    int64_t s, m, q0, t0, start, arrival;
    float eta;
};

struct Layout {
    size_t w0, Wg, W, U, loss, params, arrivals, debug, labels, fused, wgrad;
    size_t act[AET_MAX_LAYERS + 1], del[AET_MAX_LAYERS + 1], amax[AET_MAX_LAYERS];
    size_t total;
};

std::string g_init_error;

size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }


// Geometry of every layer, or false if the description is not supported.
bool resolve(const aet_model_desc *m, LayerGeom *lay, int64_t *P, std::string *why) {
    if (!m || m->n_layers < 1 || m->n_layers > AET_MAX_LAYERS) { *why = "n_layers out of range"; return false; }
    if (m->batch < 1 || m->batch > 256) { *why = "batch must be 1..256"; return false; }
    if (m->in_c < 1 || m->in_h < 1 || m->in_w < 1) { *why = "bad input shape"; return false; }
    int c = m->in_c, h = m->in_h, w = m->in_w;
    int64_t off = 0;
    for (int l = 0; l < m->n_layers; ++l) {
        const aet_layer &q = m->layers[l];
        LayerGeom &o = lay[l];
        std::memset(&o, 0, sizeof o);
        o.type = q.type; o.relu = q.relu ? 1 : 0; o.k = q.k; o.pad = q.pad;
        o.ic = c; o.ih = h; o.iw = w;
        o.in_size = (int64_t)c * h * w;
        if (q.type == AET_CONV) {
            if (!(q.k == 1 || q.k == 2 || q.k == 3 || q.k == 5)) { *why = "conv kernel size must be 1, 2, 3 or 5"; return false; }
            if (q.pad < 0 || q.pad >= q.k || q.cout < 1) { *why = "bad conv layer"; return false; }
            o.oc = q.cout; o.oh = h + 2 * q.pad - q.k + 1; o.ow = w + 2 * q.pad - q.k + 1;
            if (o.oh < 1 || o.ow < 1) { *why = "conv output is empty"; return false; }
            o.w_off = off; off += (int64_t)q.cout * c * q.k * q.k;
            o.b_off = off; off += q.cout;
        } else if (q.type == AET_POOL) {
            if ((h & 1) || (w & 1)) { *why = "pool input must have even height and width"; return false; }
            if (l == 0) { *why = "first layer cannot be a pool"; return false; }
            o.oc = c; o.oh = h / 2; o.ow = w / 2; o.relu = 0;
        } else if (q.type == AET_DENSE) {
            if (q.cout < 1) { *why = "bad dense layer"; return false; }
            o.oc = q.cout; o.oh = 1; o.ow = 1;
            o.w_off = off; off += (int64_t)q.cout * o.in_size;
            o.b_off = off; off += q.cout;
        } else { *why = "unknown layer type"; return false; }
        o.out_size = (int64_t)o.oc * o.oh * o.ow;
        if (o.in_size > (1 << 28) || o.out_size > (1 << 28)) { *why = "layer too large"; return false; }
        c = o.oc; h = o.oh; w = o.ow;
    }
    const aet_layer &last = m->layers[m->n_layers - 1];
    if (last.type != AET_DENSE || last.relu) { *why = "last layer must be dense without ReLU"; return false; }
    if (last.cout > 1024) { *why = "too many classes"; return false; }
    *P = off;
    return true;
}

// which engine runs the local rounds of this model
enum Engine { ENGINE_LAYERS = 0, ENGINE_MLP = 1, ENGINE_SOFTMAX = 2, ENGINE_LENET = 3 };

// aet_test_select_kernels: which kernel set contexts created from now on use
int g_force_layer_engine = 0, g_plain_layers = 0;

Engine pick_engine(const LayerGeom *lay, int L, int B) {
    if (g_force_layer_engine) return ENGINE_LAYERS;
    if (L == 2 && lay[0].type == AET_DENSE && lay[1].type == AET_DENSE && lay[0].relu &&
        mlp_round_supported((int)lay[0].in_size, lay[0].oc, lay[1].oc, B))
        return ENGINE_MLP;
    if (L == 1 && lay[0].type == AET_DENSE && softmax_round_supported((int)lay[0].in_size, lay[0].oc, B))
        return ENGINE_SOFTMAX;
    if (lenet_round_supported(lay, L, B)) return ENGINE_LENET;
    return ENGINE_LAYERS;
}

bool make_layout(const LayerGeom *lay, int L, int64_t P, int B, int n, int inflight, int rounds,
                 Layout *lo) {
    if (n < 1 || inflight < 1 || rounds < 1) return false;
    const size_t Ps = (size_t)((P + 63) / 64 * 64);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    lo->w0 = take(Ps * 4);
    lo->Wg = take(Ps * 4);
    lo->W = take(Ps * 4 * n);
    lo->U = take(Ps * 4 * (size_t)n * inflight);
    lo->loss = take((size_t)n * rounds * 4);
    lo->params = take((size_t)n * sizeof(RoundParams));
    lo->arrivals = take((size_t)n * inflight * sizeof(Arrival));
    lo->debug = take((size_t)kDebugIdx * 4);
    lo->labels = take((size_t)n * B * 4);
    // exchange records of the fused dense-ReLU-dense engine, only for models it runs
    const Engine eng = pick_engine(lay, L, B);
    lo->fused = take(eng == ENGINE_MLP ? mlp_round_scratch_bytes(n, B) : eng == ENGINE_LENET ? lenet_round_scratch_bytes(n) : 0);
    size_t wg_floats = 0;
    for (int l = 0; l < L; ++l)
        if (lay[l].type == AET_CONV && conv_wgrad_mfma_supported(lay[l], B))
            wg_floats = std::max(wg_floats, conv_wgrad_partial_floats(lay[l], B, n));
    lo->wgrad = take(wg_floats * 4);
    const size_t samples = (size_t)n * B;
    lo->act[0] = take(samples * lay[0].in_size * 4);
    lo->del[0] = 0;
    for (int l = 0; l < L; ++l) {
        lo->act[l + 1] = take(samples * lay[l].out_size * 4);
        lo->del[l + 1] = take(samples * lay[l].out_size * 4);
        lo->amax[l] = lay[l].type == AET_POOL ? take(samples * lay[l].out_size) : 0;
    }
    lo->total = off;
    return true;
}

}  // namespace

struct aet_ctx {
    LayerGeom lay[AET_MAX_LAYERS];
    int L = 0, B = 0, n = 0, inflight = 0, max_rounds = 0;
    int64_t P = 0, Ps = 0;
    uint64_t seed = 0;
    hipStream_t stream = nullptr;
    char *ws = nullptr;
    Layout lo{};
    LayerScratch sc{};
    std::vector<aet_shard> shards;
    std::vector<uint64_t> key;
    std::vector<int64_t> i_c, t_c, q_c, free_at, H;
    std::vector<std::vector<RoundRec>> recs;
    std::vector<Msg> queue;
    std::vector<int> free_slots;
    int64_t tick = 0;
    RoundParams *h_params[kRing] = {};
    Arrival *h_arr[kRing] = {};
    hipEvent_t ev_params[kRing] = {}, ev_arr[kRing] = {};
    int ring_p = 0, ring_a = 0;
    // a context on the library's own workspace has no pinned rings: its records reach the
    // device through kernel arguments, staged in these host vectors
    bool static_ws = false;
    int device = -1;
    std::vector<RoundParams> v_params;
    std::vector<Arrival> v_arr;
    bool dead = false;
    // peer-to-peer form: neighbour lists (host copy and device copy in the caller's buffer)
    bool p2p = false;
    std::vector<int32_t> nbr_off, nbr;
    int32_t *d_nbr_off = nullptr, *d_nbr = nullptr;
    // Setup (Algorithm 1): node weights and, per global round, every node's share of it
    bool setup = false;
    uint64_t setup_seed = 0;
    std::vector<uint64_t> cumw;
    int64_t setup_a = -1, setup_b = -1;
    std::vector<std::vector<int64_t>> setup_share;  // [round][node] recursions
    int engine = 0;
    uint32_t epoch = 0;  // step-tag base of the fused kernels' exchange records
    std::string err;
    Profiler prof;
    Profiler *profp() { return prof.any ? &prof : nullptr; }
    float *W0() const { return reinterpret_cast<float *>(ws + lo.w0); }

    float *Wg() const { return reinterpret_cast<float *>(ws + lo.Wg); }
    float *Wc(int c) const { return reinterpret_cast<float *>(ws + lo.W) + (int64_t)c * Ps; }
    float *Uslot(int s) const { return reinterpret_cast<float *>(ws + lo.U) + (int64_t)s * Ps; }
    float *loss_at(int c, int k) const {
        return reinterpret_cast<float *>(ws + lo.loss) + (int64_t)c * max_rounds + k;
    }
};

namespace {

aet_status fail(aet_ctx *ctx, aet_status st, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (ctx) ctx->err = buf; else g_init_error = buf;
    return st;
}

aet_status hip_fail(aet_ctx *ctx, hipError_t e, const char *what) {
    if (ctx) ctx->dead = true;
    return fail(ctx, AET_EHIP, "%s: %s", what, hipGetErrorString(e));
}

#define AET_HIP(ctx, call)                                   \
    do {                                                     \
        hipError_t e_ = (call);                              \
        if (e_ != hipSuccess) return hip_fail(ctx, e_, #call); \
    } while (0)

// Recursions of global round i that the coin flips of Algorithm 1 hand to every node:
// recursion t goes to the node whose cumulative-weight interval holds the t-th value of the
// hash stream of (seed, round i), mapped onto [0, sum of weights) by multiply-shift.
const std::vector<int64_t> &setup_shares(aet_ctx *ctx, int64_t i, int64_t a, int64_t b) {
    if (a != ctx->setup_a || b != ctx->setup_b) {
        ctx->setup_share.clear();
        ctx->setup_a = a;
        ctx->setup_b = b;
    }
    if ((int64_t)ctx->setup_share.size() <= i) ctx->setup_share.resize(i + 1);
    std::vector<int64_t> &sh = ctx->setup_share[i];
    if (sh.empty()) {
        sh.assign(ctx->n, 0);
        const uint64_t key = splitmix_at(splitmix_at(ctx->setup_seed, kTagSetup), (uint64_t)i);
        const uint64_t W = ctx->cumw.back();
        const int64_t steps = (a * i + b) / ctx->B;
        for (int64_t t = 0; t < steps; ++t) {
            const uint64_t r = ((splitmix_at(key, (uint64_t)t) >> 32) * W) >> 32;
            const int c = (int)(std::upper_bound(ctx->cumw.begin(), ctx->cumw.end(), r) - ctx->cumw.begin());
            sh[c] += 1;
        }
    }
    return sh;
}

}  // namespace

extern "C" {

void aet_test_select_kernels(int32_t force_layer_engine, int32_t plain_layers) {
    g_force_layer_engine = force_layer_engine != 0;
    g_plain_layers = plain_layers != 0;
}

int64_t aet_n_params(const aet_model_desc *model) {
    LayerGeom lay[AET_MAX_LAYERS];
    int64_t P;
    std::string why;
    return resolve(model, lay, &P, &why) ? P : -1;
}

size_t aet_workspace_bytes(const aet_model_desc *model, int32_t n_clients, int32_t max_inflight,
                           int32_t max_rounds) {
    LayerGeom lay[AET_MAX_LAYERS];
    int64_t P;
    std::string why;
    Layout lo;
    if (!resolve(model, lay, &P, &why)) return 0;
    if (!make_layout(lay, model->n_layers, P, model->batch, n_clients, max_inflight, max_rounds, &lo))
        return 0;
    return lo.total;
}

// Both forms of Setup.  static_ws: the workspace is the library's own array on the current
// device, w0 is a DEVICE pointer, and nothing is allocated with HIP (no pinned rings, no
// events).
static aet_status init_context(aet_ctx **out, const aet_model_desc *model, int32_t n_clients,
                               const aet_shard *shards, const float *w0, uint64_t seed, void *workspace,
                               size_t workspace_bytes, int32_t max_inflight, int32_t max_rounds,
                               void *hip_stream, bool static_ws) {
    if (!out) return fail(nullptr, AET_EINVAL, "out is NULL");
    *out = nullptr;
    if (!model || !shards || !w0 || (!workspace && !static_ws)) return fail(nullptr, AET_EINVAL, "NULL argument");
    if (n_clients < 1 || n_clients > 65535) return fail(nullptr, AET_EINVAL, "n_clients must be 1..65535");
    if (max_inflight < 1 || max_rounds < 1) return fail(nullptr, AET_EINVAL, "max_inflight and max_rounds must be >= 1");
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return fail(nullptr, AET_EINVAL, "workspace must be 256-byte aligned");
    int dev = -1;
    if (static_ws) {
        // the library's array on the current device: its address once per device, one
        // context at a time
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return fail(nullptr, AET_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
        if (dev < 0 || dev >= kMaxDevices) return fail(nullptr, AET_EINVAL, "device ordinal %d not supported", dev);
        if (g_scratch_owner[dev])
            return fail(nullptr, AET_ESTATE, "the library's workspace on device %d belongs to a live context: destroy it first", dev);
        e = scratch_address(dev, &workspace);
        if (e != hipSuccess) return fail(nullptr, AET_EHIP, "hipGetSymbolAddress: %s", hipGetErrorString(e));
        workspace_bytes = kStaticBytes;
    }
    aet_ctx *ctx = new (std::nothrow) aet_ctx();
    if (!ctx) return fail(nullptr, AET_ENOMEM, "host allocation failed");
    ctx->static_ws = static_ws;
    ctx->device = dev;
    std::string why;
    if (!resolve(model, ctx->lay, &ctx->P, &why)) {
        delete ctx;
        return fail(nullptr, AET_EINVAL, "unsupported model: %s", why.c_str());
    }
    ctx->L = model->n_layers; ctx->B = model->batch; ctx->n = n_clients;
    ctx->inflight = max_inflight; ctx->max_rounds = max_rounds;
    ctx->Ps = (ctx->P + 63) / 64 * 64;
    ctx->seed = seed;
    ctx->stream = reinterpret_cast<hipStream_t>(hip_stream);
    ctx->ws = static_cast<char *>(workspace);
    make_layout(ctx->lay, ctx->L, ctx->P, ctx->B, ctx->n, max_inflight, max_rounds, &ctx->lo);
    if (workspace_bytes < ctx->lo.total) {
        const size_t need = ctx->lo.total;
        delete ctx;
        if (static_ws)
            return fail(nullptr, AET_ENOMEM, "this model and client count need %zu bytes of workspace, the library's own holds %zu: use aet_init with a workspace of your own", need, workspace_bytes);
        return fail(nullptr, AET_ENOMEM, "workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);
    }
    for (int c = 0; c < n_clients; ++c) {
        if (!shards[c].X || !shards[c].y || shards[c].n_samples < 1 || shards[c].n_samples > 2147483647LL) {
            delete ctx;
            return fail(nullptr, AET_EINVAL, "shard %d: NULL pointer or n_samples outside 1..2^31-1", c);
        }
    }
    ctx->shards.assign(shards, shards + n_clients);
    ctx->key.resize(n_clients);
    const uint64_t sample_key = splitmix_at(seed, kTagSample);
    for (int c = 0; c < n_clients; ++c) ctx->key[c] = splitmix_at(sample_key, (uint64_t)c);
    ctx->i_c.assign(n_clients, 0); ctx->t_c.assign(n_clients, 0); ctx->q_c.assign(n_clients, 0);
    ctx->free_at.assign(n_clients, 0); ctx->H.assign(n_clients, 0);
    ctx->recs.resize(n_clients);
    for (int s = n_clients * max_inflight - 1; s >= 0; --s) ctx->free_slots.push_back(s);
    for (int l = 0; l <= ctx->L; ++l) {
        ctx->sc.act[l] = reinterpret_cast<float *>(ctx->ws + ctx->lo.act[l]);
        ctx->sc.del[l] = l ? reinterpret_cast<float *>(ctx->ws + ctx->lo.del[l]) : nullptr;
    }
    for (int l = 0; l < ctx->L; ++l)
        ctx->sc.amax[l] = ctx->lay[l].type == AET_POOL ? reinterpret_cast<uint8_t *>(ctx->ws + ctx->lo.amax[l]) : nullptr;
    ctx->sc.labels = reinterpret_cast<int32_t *>(ctx->ws + ctx->lo.labels);
    ctx->sc.wgrad = reinterpret_cast<float *>(ctx->ws + ctx->lo.wgrad);
    ctx->sc.plain = g_plain_layers != 0;
    ctx->engine = pick_engine(ctx->lay, ctx->L, ctx->B);

    hipError_t e = hipSuccess;
    if (static_ws) {
        // the array keeps what the last context left: everything this one will use starts at zero
        const size_t n16 = (ctx->lo.total + 15) / 16;
        k_clear_bytes16<<<(unsigned)((n16 + 255) / 256), 256, 0, ctx->stream>>>(reinterpret_cast<uint4 *>(ctx->ws), n16);
        e = hipGetLastError();
        ctx->v_params.resize(n_clients);
        ctx->v_arr.resize((size_t)n_clients * max_inflight);
    }
    for (int r = 0; r < kRing && e == hipSuccess && !static_ws; ++r) {
        e = hipHostMalloc(reinterpret_cast<void **>(&ctx->h_params[r]), (size_t)n_clients * sizeof(RoundParams), hipHostMallocDefault);
        if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void **>(&ctx->h_arr[r]), (size_t)n_clients * max_inflight * sizeof(Arrival), hipHostMallocDefault);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_params[r], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_arr[r], hipEventDisableTiming);
    }
    if (e == hipSuccess && ctx->engine == ENGINE_MLP)
        e = mlp_clear_error_flag(ctx->stream, ctx->ws + ctx->lo.fused, n_clients, ctx->B);
    if (e == hipSuccess && ctx->engine == ENGINE_LENET)
        e = lenet_clear_error_flag(ctx->stream, ctx->ws + ctx->lo.fused, n_clients);
    // global model and every replica start as w0
    if (e == hipSuccess) e = hipMemcpyAsync(ctx->W0(), w0, (size_t)ctx->P * 4, static_ws ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);  // w0 is the caller's; do not keep reading it
    if (e == hipSuccess) e = hipMemcpyAsync(ctx->Wg(), ctx->W0(), (size_t)ctx->P * 4, hipMemcpyDeviceToDevice, ctx->stream);
    if (e == hipSuccess) e = launch_broadcast_model(ctx->stream, ctx->Wc(0), ctx->Ps, n_clients, ctx->W0());
    if (e != hipSuccess) {
        const aet_status st = fail(nullptr, AET_EHIP, "aet_init: %s", hipGetErrorString(e));
        aet_destroy(ctx);
        return st;
    }
    if (static_ws) g_scratch_owner[dev] = ctx;
    *out = ctx;
    return AET_OK;
}

aet_status aet_init(aet_ctx **out, const aet_model_desc *model, int32_t n_clients,
                    const aet_shard *shards, const float *w0, uint64_t seed, void *workspace,
                    size_t workspace_bytes, int32_t max_inflight, int32_t max_rounds,
                    void *hip_stream) {
    return init_context(out, model, n_clients, shards, w0, seed, workspace, workspace_bytes,
                        max_inflight, max_rounds, hip_stream, false);
}

aet_status aet_init_static(aet_ctx **out, const aet_model_desc *model, int32_t n_clients,
                           const aet_shard *shards, const float *w0_dev, uint64_t seed,
                           int32_t max_inflight, int32_t max_rounds, void *hip_stream) {
    return init_context(out, model, n_clients, shards, w0_dev, seed, nullptr, 0, max_inflight,
                        max_rounds, hip_stream, true);
}

aet_status aet_run_round(aet_ctx *ctx, const aet_threshold *thr, const aet_eta *eta,
                         const aet_delay *delay, int32_t *n_finished, int32_t *finished_client,
                         int32_t *finished_round) {
    if (!ctx) return AET_EINVAL;
    if (ctx->dead) return fail(ctx, AET_ESTATE, "context is unusable after a HIP error");
    if (!thr || !eta) return fail(ctx, AET_EINVAL, "NULL argument");
    if (thr->a < 0 || thr->b < 0 || thr->rounds < 0) return fail(ctx, AET_EINVAL, "threshold parameters must be non-negative");
    if (thr->rounds > ctx->max_rounds) return fail(ctx, AET_EINVAL, "rounds exceeds max_rounds given to aet_init");
    if (!(eta->eta0 > 0) || eta->beta < 0 || !std::isfinite(eta->eta0) || !std::isfinite(eta->beta) || !std::isfinite(eta->power))
        return fail(ctx, AET_EINVAL, "bad step size parameters");
    const int32_t dmin = delay ? delay->delay_min : 0, dmax = delay ? delay->delay_max : 0;
    if (dmin < 0 || dmax < dmin || dmax >= ctx->inflight)
        return fail(ctx, AET_EINVAL, "need 0 <= delay_min <= delay_max < max_inflight");
    const int32_t *cf = delay ? delay->compute_factor : nullptr;
    const uint8_t *st = delay ? delay->is_straggler : nullptr;
    const int32_t d_gate = delay ? delay->d_max : -1;

    // which clients run a round this tick (ascending), and with what
    std::vector<int> act;
    std::vector<RoundRec> rec;
    int64_t max_m = 0;
    for (int c = 0; c < ctx->n; ++c) {
        if (ctx->free_at[c] > ctx->tick || ctx->i_c[c] >= thr->rounds) continue;
        if (d_gate >= 0) {  // Synchronize: d_c = max over the map H of (i - H_e)
            int64_t dc = 0;
            if (ctx->p2p) {  // the map holds the neighbours
                for (int32_t j = ctx->nbr_off[c]; j < ctx->nbr_off[c + 1]; ++j)
                    dc = std::max(dc, ctx->i_c[c] - ctx->H[ctx->nbr[j]]);
            } else {         // the map holds every other node
                for (int e = 0; e < ctx->n; ++e)
                    if (e != c) dc = std::max(dc, ctx->i_c[c] - ctx->H[e]);
            }
            if (dc > d_gate) continue;
        }
        if (cf && cf[c] < 1) return fail(ctx, AET_EINVAL, "compute_factor[%d] < 1", c);
        const int64_t i = ctx->i_c[c];
        int64_t s = thr->a * i + thr->b;
        if (s % ctx->B) return fail(ctx, AET_EINVAL, "round length s_%lld = %lld of client %d is not a multiple of batch %d", (long long)i, (long long)s, c, ctx->B);
        if (ctx->setup) s = setup_shares(ctx, i, thr->a, thr->b)[c] * ctx->B;  // s_{i,c} of Algorithm 1
        const int64_t m = s / ctx->B;
        if (m > 2147483647LL) return fail(ctx, AET_EINVAL, "round too long");
        RoundRec r;
        r.s = s; r.m = m; r.q0 = ctx->q_c[c]; r.t0 = ctx->t_c[c]; r.start = ctx->tick;
        r.eta = (float)(eta->eta0 / (1.0 + eta->beta * std::pow((double)ctx->t_c[c], eta->power)));
        const int64_t f = cf ? cf[c] : 1;
        int64_t delta = 0;
        if (st && st[c]) {
            const uint64_t h = splitmix_at(splitmix_at(splitmix_at(delay->seed, kTagNet), (uint64_t)c), (uint64_t)i);
            delta = dmin + (int64_t)(((h >> 32) * (uint64_t)(dmax - dmin + 1)) >> 32);
        }
        r.arrival = ctx->tick + f - 1 + delta;
        act.push_back(c);
        rec.push_back(r);
        max_m = std::max(max_m, m);
    }
    const int nact = (int)act.size();
    if ((int)ctx->free_slots.size() < nact)
        return fail(ctx, AET_ENOMEM, "no free U slot: more than max_inflight messages of a client in flight");

    if (nact > 0) {
        // staging: the layer engine copies the records to the device from a pinned ring; the
        // dense-ReLU-dense engine takes them in its kernel arguments from plain host memory; the
        // other two fused engines read them where they are, in the pinned ring (every workgroup
        // reads its own record once, at its start: no copy in the stream ahead of the kernel)
        const bool direct = !ctx->static_ws && (ctx->engine == ENGINE_SOFTMAX || ctx->engine == ENGINE_LENET);
        const int ring = ctx->ring_p;
        RoundParams *hp = ctx->static_ws ? ctx->v_params.data() : ctx->h_params[ring];
        if (ctx->engine != ENGINE_MLP && !ctx->static_ws) {
            ctx->ring_p = (ring + 1) % kRing;
            AET_HIP(ctx, hipEventSynchronize(ctx->ev_params[ring]));
        }
        std::vector<int> slots(nact);
        for (int a = 0; a < nact; ++a) {
            const int c = act[a];
            slots[a] = ctx->free_slots.back();
            ctx->free_slots.pop_back();
            RoundParams &p = hp[a];
            p.X = ctx->shards[c].X; p.y = ctx->shards[c].y;
            p.W = ctx->Wc(c); p.U = ctx->Uslot(slots[a]);
            p.loss = ctx->loss_at(c, (int)ctx->i_c[c]);
            p.key = ctx->key[c]; p.q0 = rec[a].q0; p.n_samples = (uint32_t)ctx->shards[c].n_samples;
            p.m = (int32_t)rec[a].m; p.eta = rec[a].eta; p.client = c;
        }
        RoundParams *dp = hp;
        if (ctx->engine != ENGINE_MLP) {
            dp = reinterpret_cast<RoundParams *>(ctx->ws + ctx->lo.params);
            if (direct) {
                dp = hp;
            } else if (ctx->static_ws) {
                for (int a0 = 0; a0 < nact; a0 += kPutParams) {
                    const int here = std::min(kPutParams, nact - a0);
                    ParamsPut put;
                    std::memcpy(put.p, hp + a0, (size_t)here * sizeof(RoundParams));
                    k_put_params<<<1, 64, 0, ctx->stream>>>(put, here, dp + a0);
                    AET_HIP(ctx, hipGetLastError());
                }
            } else {
                AET_HIP(ctx, hipMemcpyAsync(dp, hp, (size_t)nact * sizeof(RoundParams), hipMemcpyHostToDevice, ctx->stream));
                AET_HIP(ctx, hipEventRecord(ctx->ev_params[ring], ctx->stream));
            }
        }
        // server form: every round starts from the global model; peer-to-peer form: from the
        // client's own replica
        const float *start = ctx->p2p ? nullptr : ctx->Wg();
        if (ctx->engine == ENGINE_MLP) {
            AET_HIP(ctx, launch_mlp_round(ctx->stream, ctx->profp(), dp, nact, (int)max_m, start, (int)ctx->lay[0].in_size,
                                          ctx->lay[0].oc, ctx->lay[1].oc, ctx->B, ctx->ws + ctx->lo.fused, ctx->n, &ctx->epoch));
        } else if (ctx->engine == ENGINE_SOFTMAX) {
            AET_HIP(ctx, launch_softmax_round(ctx->stream, ctx->profp(), dp, nact, start, (int)ctx->lay[0].in_size, ctx->lay[0].oc));
        } else if (ctx->engine == ENGINE_LENET) {
            AET_HIP(ctx, launch_lenet_round(ctx->stream, ctx->profp(), dp, nact, (int)max_m, start, ctx->lay, ctx->L, ctx->B,
                                            ctx->ws + ctx->lo.fused, ctx->n, &ctx->epoch));
        } else {
            AET_HIP(ctx, launch_begin_round(ctx->stream, ctx->profp(), dp, nact, start, ctx->P));
            for (int64_t u = 0; u < max_m; ++u)
                AET_HIP(ctx, launch_layer_step(ctx->stream, ctx->profp(), dp, nact, (int)u, ctx->lay, ctx->L, ctx->B, ctx->sc));
        }
        if (direct) AET_HIP(ctx, hipEventRecord(ctx->ev_params[ring], ctx->stream));   // the ring slot is free after the kernel
        for (int a = 0; a < nact; ++a) {
            const int c = act[a];
            Msg msg;
            msg.c = c; msg.k = (int32_t)ctx->i_c[c]; msg.eta = rec[a].eta; msg.arrival = rec[a].arrival;
            msg.slot = slots[a];
            ctx->queue.push_back(msg);
            ctx->recs[c].push_back(rec[a]);
            ctx->t_c[c] += rec[a].m; ctx->q_c[c] += rec[a].s; ctx->i_c[c] += 1;
            ctx->free_at[c] = ctx->tick + (cf ? cf[c] : 1);
            if (finished_client) finished_client[a] = c;
            if (finished_round) finished_round[a] = msg.k;
        }
    }
    if (n_finished) *n_finished = nact;
    return AET_OK;
}

// This tick's arrivals in (round, client) order, staged for a kernel: by value when the
// list is short (*pack_out = &pack), else through the pinned ring into device memory (*dev_out).
static aet_status stage_arrivals(aet_ctx *ctx, float scale, std::vector<Msg> *arr_out, ArrivalPack *pack,
                                 const ArrivalPack **pack_out, const Arrival **dev_out) {
    std::vector<Msg> &arr = *arr_out;
    arr.clear();
    for (const Msg &m : ctx->queue)
        if (m.arrival == ctx->tick) arr.push_back(m);
    std::sort(arr.begin(), arr.end(), [](const Msg &x, const Msg &y) { return x.k != y.k ? x.k < y.k : x.c < y.c; });
    const int na = (int)arr.size();
    *pack_out = nullptr;
    *dev_out = nullptr;
    if (na == 0) return AET_OK;
    Arrival *dst = pack->a;
    int ring = -1;
    if (na > kArrivalPack && ctx->static_ws) {
        ring = kRing;  // no ring: staged in host memory, handed over in kernel arguments
        dst = ctx->v_arr.data();
    } else if (na > kArrivalPack) {
        ring = ctx->ring_a;
        ctx->ring_a = (ring + 1) % kRing;
        AET_HIP(ctx, hipEventSynchronize(ctx->ev_arr[ring]));
        dst = ctx->h_arr[ring];
    }
    for (int j = 0; j < na; ++j) {
        dst[j].U = ctx->Uslot(arr[j].slot);
        dst[j].scale = (float)((double)scale * (double)arr[j].eta);
        dst[j].sender = arr[j].c;
    }
    if (ring < 0) {
        *pack_out = pack;
    } else {
        Arrival *da = reinterpret_cast<Arrival *>(ctx->ws + ctx->lo.arrivals);
        if (ring == kRing) {
            for (int a0 = 0; a0 < na; a0 += kPutArrivals) {
                const int here = std::min(kPutArrivals, na - a0);
                ArrivalsPut put;
                std::memcpy(put.a, dst + a0, (size_t)here * sizeof(Arrival));
                k_put_arrivals<<<1, 256, 0, ctx->stream>>>(put, here, da + a0);
                AET_HIP(ctx, hipGetLastError());
            }
        } else {
            AET_HIP(ctx, hipMemcpyAsync(da, dst, (size_t)na * sizeof(Arrival), hipMemcpyHostToDevice, ctx->stream));
            AET_HIP(ctx, hipEventRecord(ctx->ev_arr[ring], ctx->stream));
        }
        *dev_out = da;
    }
    return AET_OK;
}

// bookkeeping after the arrivals were applied: H, slots, queue, outputs, tick
static void retire_arrivals(aet_ctx *ctx, const std::vector<Msg> &arr, int32_t *n_applied,
                            int32_t *applied_client, int32_t *applied_round) {
    const int na = (int)arr.size();
    for (int j = 0; j < na; ++j) {
        ctx->H[arr[j].c] += 1;
        ctx->free_slots.push_back(arr[j].slot);
        if (applied_client) applied_client[j] = arr[j].c;
        if (applied_round) applied_round[j] = arr[j].k;
    }
    if (na > 0) {
        const int64_t now = ctx->tick;
        ctx->queue.erase(std::remove_if(ctx->queue.begin(), ctx->queue.end(), [now](const Msg &m) { return m.arrival == now; }), ctx->queue.end());
    }
    if (n_applied) *n_applied = na;
    ctx->tick += 1;
}

aet_status aet_server_aggregate(aet_ctx *ctx, float agg_scale, int32_t *n_applied,
                                int32_t *applied_client, int32_t *applied_round) {
    if (!ctx) return AET_EINVAL;
    if (ctx->dead) return fail(ctx, AET_ESTATE, "context is unusable after a HIP error");
    if (ctx->p2p) return fail(ctx, AET_ESTATE, "a topology is set: the tick's second half is aet_receive");
    if (!std::isfinite(agg_scale)) return fail(ctx, AET_EINVAL, "agg_scale is not finite");
    std::vector<Msg> arr;
    ArrivalPack pack;
    const ArrivalPack *by_value = nullptr;
    const Arrival *on_device = nullptr;
    const aet_status st = stage_arrivals(ctx, agg_scale, &arr, &pack, &by_value, &on_device);
    if (st != AET_OK) return st;
    const int na = (int)arr.size();
    if (by_value) {
        AET_HIP(ctx, launch_server_apply_small(ctx->stream, ctx->profp(), ctx->Wg(), *by_value, na, ctx->P));
    } else if (on_device) {
        AET_HIP(ctx, launch_server_reduce(ctx->stream, ctx->profp(), ctx->Wg(), on_device, na, ctx->P));
    }
    retire_arrivals(ctx, arr, n_applied, applied_client, applied_round);
    return AET_OK;
}

aet_status aet_set_setup(aet_ctx *ctx, const uint32_t *weights, uint64_t seed) {
    if (!ctx) return AET_EINVAL;
    if (!weights) return fail(ctx, AET_EINVAL, "NULL argument");
    for (int c = 0; c < ctx->n; ++c)
        if (ctx->i_c[c] != 0) return fail(ctx, AET_ESTATE, "Setup comes before the first round");
    uint64_t sum = 0;
    for (int c = 0; c < ctx->n; ++c) sum += weights[c];
    if (sum < 1 || sum >= (1ull << 32)) return fail(ctx, AET_EINVAL, "the sum of the weights must be in [1, 2^32)");
    ctx->cumw.resize(ctx->n);
    sum = 0;
    for (int c = 0; c < ctx->n; ++c) { sum += weights[c]; ctx->cumw[c] = sum; }
    ctx->setup = true;
    ctx->setup_seed = seed;
    ctx->setup_share.clear();
    return AET_OK;
}

size_t aet_topology_workspace_bytes(int32_t n_clients, int32_t n_neighbour_entries) {
    if (n_clients < 1 || n_neighbour_entries < 0) return 0;
    return align_up((size_t)(n_clients + 1) * 4) + align_up((size_t)std::max(n_neighbour_entries, 1) * 4);
}

aet_status aet_set_topology(aet_ctx *ctx, const int32_t *nbr_off, const int32_t *nbr, void *workspace,
                            size_t workspace_bytes) {
    if (!ctx) return AET_EINVAL;
    if (ctx->dead) return fail(ctx, AET_ESTATE, "context is unusable after a HIP error");
    if (!nbr_off || !workspace) return fail(ctx, AET_EINVAL, "NULL argument");
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return fail(ctx, AET_EINVAL, "workspace must be 256-byte aligned");
    if (ctx->tick != 0 || !ctx->queue.empty()) return fail(ctx, AET_ESTATE, "the topology must be set before the first round");
    for (int c = 0; c < ctx->n; ++c)
        if (ctx->i_c[c] != 0) return fail(ctx, AET_ESTATE, "the topology must be set before the first round");
    const int n = ctx->n;
    if (nbr_off[0] != 0) return fail(ctx, AET_EINVAL, "nbr_off[0] must be 0");
    for (int c = 0; c < n; ++c)
        if (nbr_off[c + 1] < nbr_off[c]) return fail(ctx, AET_EINVAL, "nbr_off must not decrease");
    const int32_t E = nbr_off[n];
    if (E > 0 && !nbr) return fail(ctx, AET_EINVAL, "NULL argument");
    for (int c = 0; c < n; ++c)
        for (int32_t j = nbr_off[c]; j < nbr_off[c + 1]; ++j) {
            const int32_t v = nbr[j];
            if (v < 0 || v >= n || v == c) return fail(ctx, AET_EINVAL, "node %d: neighbour %d out of range or the node itself", c, v);
            if (j > nbr_off[c] && nbr[j - 1] >= v) return fail(ctx, AET_EINVAL, "node %d: neighbours must be strictly ascending", c);
        }
    // every list is sorted now, so the reverse edge can be looked up by bisection
    for (int c = 0; c < n; ++c)
        for (int32_t j = nbr_off[c]; j < nbr_off[c + 1]; ++j) {
            const int32_t v = nbr[j];
            if (!std::binary_search(nbr + nbr_off[v], nbr + nbr_off[v + 1], (int32_t)c))
                return fail(ctx, AET_EINVAL, "topology is not undirected: %d lists %d but not the reverse", c, v);
        }
    const size_t need = aet_topology_workspace_bytes(n, E);
    if (workspace_bytes < need) return fail(ctx, AET_ENOMEM, "topology workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);
    ctx->nbr_off.assign(nbr_off, nbr_off + n + 1);
    ctx->nbr.assign(nbr, nbr + E);
    ctx->d_nbr_off = static_cast<int32_t *>(workspace);
    ctx->d_nbr = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + align_up((size_t)(n + 1) * 4));
    // the host copies above outlive the call, so the asynchronous uploads may read them
    AET_HIP(ctx, hipMemcpyAsync(ctx->d_nbr_off, ctx->nbr_off.data(), (size_t)(n + 1) * 4, hipMemcpyHostToDevice, ctx->stream));
    if (E > 0) AET_HIP(ctx, hipMemcpyAsync(ctx->d_nbr, ctx->nbr.data(), (size_t)E * 4, hipMemcpyHostToDevice, ctx->stream));
    AET_HIP(ctx, hipStreamSynchronize(ctx->stream));
    ctx->p2p = true;
    return AET_OK;
}

aet_status aet_receive(aet_ctx *ctx, float scale, int32_t *n_applied, int32_t *applied_sender,
                       int32_t *applied_round) {
    if (!ctx) return AET_EINVAL;
    if (ctx->dead) return fail(ctx, AET_ESTATE, "context is unusable after a HIP error");
    if (!ctx->p2p) return fail(ctx, AET_ESTATE, "no topology set: the tick's second half is aet_server_aggregate");
    if (!std::isfinite(scale)) return fail(ctx, AET_EINVAL, "scale is not finite");
    std::vector<Msg> arr;
    ArrivalPack pack;
    const ArrivalPack *by_value = nullptr;
    const Arrival *on_device = nullptr;
    const aet_status st = stage_arrivals(ctx, scale, &arr, &pack, &by_value, &on_device);
    if (st != AET_OK) return st;
    if (by_value || on_device)
        AET_HIP(ctx, launch_apply_neighbour_U(ctx->stream, ctx->profp(), ctx->Wc(0), ctx->Ps, ctx->P, ctx->n,
                                              ctx->d_nbr_off, ctx->d_nbr, by_value, on_device, (int)arr.size()));
    retire_arrivals(ctx, arr, n_applied, applied_sender, applied_round);
    return AET_OK;
}

// After a synchronisation: did a fused kernel give up waiting for its cluster peers?
static aet_status check_device_flag(aet_ctx *ctx) {
    if (ctx->engine != ENGINE_MLP && ctx->engine != ENGINE_LENET) return AET_OK;
    int flag = 0;
    const int *dflag = ctx->engine == ENGINE_MLP ? mlp_error_flag_ptr(ctx->ws + ctx->lo.fused, ctx->n, ctx->B)
                                                 : lenet_error_flag_ptr(ctx->ws + ctx->lo.fused, ctx->n);
    AET_HIP(ctx, hipMemcpyAsync(&flag, dflag, 4, hipMemcpyDeviceToHost, ctx->stream));
    AET_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (flag) {
        ctx->dead = true;
        return fail(ctx, AET_EHIP, "a fused round kernel timed out in its cluster barrier; results are invalid");
    }
    return AET_OK;
}

aet_status aet_run_ticks(aet_ctx *ctx, const aet_threshold *thr, const aet_eta *eta,
                         const aet_delay *delay, float agg_scale, int32_t max_ticks,
                         int32_t *ticks_done) {
    if (!ctx) return AET_EINVAL;
    if (!thr) return fail(ctx, AET_EINVAL, "NULL argument");
    int32_t done = 0;
    if (ticks_done) *ticks_done = 0;
    while (done < max_ticks && !aet_all_done(ctx, thr->rounds)) {
        aet_status st = aet_run_round(ctx, thr, eta, delay, nullptr, nullptr, nullptr);
        if (st != AET_OK) return st;
        st = ctx->p2p ? aet_receive(ctx, agg_scale, nullptr, nullptr, nullptr)
                      : aet_server_aggregate(ctx, agg_scale, nullptr, nullptr, nullptr);
        if (st != AET_OK) return st;
        ++done;
        if (ticks_done) *ticks_done = done;
    }
    return AET_OK;
}

static aet_status copy_out(aet_ctx *ctx, const float *src, float *dst, int32_t on_host) {
    if (on_host) {
        AET_HIP(ctx, hipMemcpyAsync(dst, src, (size_t)ctx->P * 4, hipMemcpyDeviceToHost, ctx->stream));
        AET_HIP(ctx, hipStreamSynchronize(ctx->stream));
        return check_device_flag(ctx);
    } else {
        AET_HIP(ctx, hipMemcpyAsync(dst, src, (size_t)ctx->P * 4, hipMemcpyDeviceToDevice, ctx->stream));
    }
    return AET_OK;
}

aet_status aet_get_U(aet_ctx *ctx, int32_t client, int32_t round, float *dst, int32_t on_host) {
    if (!ctx) return AET_EINVAL;
    if (ctx->dead) return fail(ctx, AET_ESTATE, "context is unusable after a HIP error");
    if (!dst) return fail(ctx, AET_EINVAL, "dst is NULL");
    for (const Msg &m : ctx->queue)
        if (m.c == client && m.k == round) return copy_out(ctx, ctx->Uslot(m.slot), dst, on_host);
    return fail(ctx, AET_ESTATE, "message (client %d, round %d) is not in flight", client, round);
}

aet_status aet_get_weights(aet_ctx *ctx, int32_t client, float *dst, int32_t on_host) {
    if (!ctx) return AET_EINVAL;
    if (ctx->dead) return fail(ctx, AET_ESTATE, "context is unusable after a HIP error");
    if (!dst) return fail(ctx, AET_EINVAL, "dst is NULL");
    if (client >= ctx->n) return fail(ctx, AET_EINVAL, "client out of range");
    return copy_out(ctx, client < 0 ? ctx->Wg() : ctx->Wc(client), dst, on_host);
}

aet_status aet_set_weights(aet_ctx *ctx, int32_t client, const float *src, int32_t on_host) {
    if (!ctx) return AET_EINVAL;
    if (ctx->dead) return fail(ctx, AET_ESTATE, "context is unusable after a HIP error");
    if (!src) return fail(ctx, AET_EINVAL, "src is NULL");
    if (client >= ctx->n) return fail(ctx, AET_EINVAL, "client out of range");
    float *dst = client < 0 ? ctx->Wg() : ctx->Wc(client);
    AET_HIP(ctx, hipMemcpyAsync(dst, src, (size_t)ctx->P * 4, on_host ? hipMemcpyHostToDevice : hipMemcpyDeviceToDevice, ctx->stream));
    if (on_host) AET_HIP(ctx, hipStreamSynchronize(ctx->stream));  // src is the caller's: done with it on return
    return AET_OK;
}

aet_status aet_get_round_info(aet_ctx *ctx, int32_t client, int32_t round, int64_t *ints,
                              double *dbls) {
    if (!ctx) return AET_EINVAL;
    if (client < 0 || client >= ctx->n || round < 0 || round >= (int)ctx->recs[client].size())
        return fail(ctx, AET_ESTATE, "client %d has not run round %d", client, round);
    if (ctx->dead) return fail(ctx, AET_ESTATE, "context is unusable after a HIP error");
    const RoundRec &r = ctx->recs[client][round];
    if (ints) { ints[0] = r.s; ints[1] = r.m; ints[2] = r.q0; ints[3] = r.t0; ints[4] = r.start; ints[5] = r.arrival; }
    if (dbls) {
        float loss = 0.f;
        AET_HIP(ctx, hipMemcpyAsync(&loss, ctx->loss_at(client, round), 4, hipMemcpyDeviceToHost, ctx->stream));
        AET_HIP(ctx, hipStreamSynchronize(ctx->stream));
        const aet_status st = check_device_flag(ctx);
        if (st != AET_OK) return st;
        dbls[0] = (double)r.eta;
        dbls[1] = r.m > 0 ? (double)loss / (double)r.m : 0.0;
    }
    return AET_OK;
}

aet_status aet_debug_sample_indices(aet_ctx *ctx, int32_t client, int64_t q0, int32_t count,
                                    int32_t *dst) {
    if (!ctx) return AET_EINVAL;
    if (ctx->dead) return fail(ctx, AET_ESTATE, "context is unusable after a HIP error");
    if (client < 0 || client >= ctx->n || q0 < 0 || count < 0 || count > kDebugIdx || !dst)
        return fail(ctx, AET_EINVAL, "bad argument");
    if (count == 0) return AET_OK;
    int32_t *d = reinterpret_cast<int32_t *>(ctx->ws + ctx->lo.debug);
    AET_HIP(ctx, launch_debug_indices(ctx->stream, ctx->key[client], q0, count, (uint32_t)ctx->shards[client].n_samples, d));
    AET_HIP(ctx, hipMemcpyAsync(dst, d, (size_t)count * 4, hipMemcpyDeviceToHost, ctx->stream));
    AET_HIP(ctx, hipStreamSynchronize(ctx->stream));
    return AET_OK;
}

int32_t aet_all_done(const aet_ctx *ctx, int32_t rounds) {
    if (!ctx || !ctx->queue.empty()) return 0;
    for (int c = 0; c < ctx->n; ++c)
        if (ctx->i_c[c] < rounds) return 0;
    return 1;
}

int64_t aet_tick(const aet_ctx *ctx) { return ctx ? ctx->tick : -1; }
int64_t aet_history(const aet_ctx *ctx, int32_t client) {
    return (ctx && client >= 0 && client < ctx->n) ? ctx->H[client] : -1;
}
int64_t aet_inflight(const aet_ctx *ctx) { return ctx ? (int64_t)ctx->queue.size() : -1; }

aet_status aet_synchronize(aet_ctx *ctx) {
    if (!ctx) return AET_EINVAL;
    AET_HIP(ctx, hipStreamSynchronize(ctx->stream));
    return check_device_flag(ctx);
}

aet_status aet_reset(aet_ctx *ctx) {
    if (!ctx) return AET_EINVAL;
    if (ctx->dead) return fail(ctx, AET_ESTATE, "context is unusable after a HIP error");
    // server form: the replicas need no copy, every round starts by adopting the global model
    AET_HIP(ctx, hipMemcpyAsync(ctx->Wg(), ctx->W0(), (size_t)ctx->P * 4, hipMemcpyDeviceToDevice, ctx->stream));
    if (ctx->p2p) AET_HIP(ctx, launch_broadcast_model(ctx->stream, ctx->Wc(0), ctx->Ps, ctx->n, ctx->W0()));
    std::fill(ctx->i_c.begin(), ctx->i_c.end(), 0);
    std::fill(ctx->t_c.begin(), ctx->t_c.end(), 0);
    std::fill(ctx->q_c.begin(), ctx->q_c.end(), 0);
    std::fill(ctx->free_at.begin(), ctx->free_at.end(), 0);
    std::fill(ctx->H.begin(), ctx->H.end(), 0);
    for (auto &r : ctx->recs) r.clear();
    ctx->queue.clear();
    ctx->free_slots.clear();
    for (int s = ctx->n * ctx->inflight - 1; s >= 0; --s) ctx->free_slots.push_back(s);
    ctx->tick = 0;
    return AET_OK;
}

int32_t aet_profile_families(void) { return F_COUNT; }
const char *aet_profile_family_name(int32_t family) { return family_name(family); }

aet_status aet_profile_enable(aet_ctx *ctx, int32_t family, int32_t on) {
    if (!ctx) return AET_EINVAL;
    if (family >= F_COUNT) return fail(ctx, AET_EINVAL, "no such kernel family");
    for (int f = 0; f < F_COUNT; ++f)
        if (family < 0 || f == family) ctx->prof.on[f] = on != 0;
    ctx->prof.any = false;
    for (int f = 0; f < F_COUNT; ++f) ctx->prof.any = ctx->prof.any || ctx->prof.on[f];
    return AET_OK;
}

aet_status aet_profile_read(aet_ctx *ctx, int32_t family, int64_t *launches, double *total_ms,
                            int32_t reset) {
    if (!ctx) return AET_EINVAL;
    if (family < 0 || family >= F_COUNT) return fail(ctx, AET_EINVAL, "no such kernel family");
    AET_HIP(ctx, ctx->prof.drain(ctx->stream));
    if (launches) *launches = ctx->prof.launches[family];
    if (total_ms) *total_ms = ctx->prof.total_ms[family];
    if (reset) { ctx->prof.launches[family] = 0; ctx->prof.total_ms[family] = 0.0; }
    return AET_OK;
}

const char *aet_last_error(const aet_ctx *ctx) { return ctx ? ctx->err.c_str() : g_init_error.c_str(); }

void aet_destroy(aet_ctx *ctx) {
    if (!ctx) return;
    (void)hipStreamSynchronize(ctx->stream);
    if (ctx->static_ws && ctx->device >= 0 && g_scratch_owner[ctx->device] == ctx) g_scratch_owner[ctx->device] = nullptr;
    for (int r = 0; r < kRing; ++r) {
        if (ctx->h_params[r]) (void)hipHostFree(ctx->h_params[r]);
        if (ctx->h_arr[r]) (void)hipHostFree(ctx->h_arr[r]);
        if (ctx->ev_params[r]) (void)hipEventDestroy(ctx->ev_params[r]);
        if (ctx->ev_arr[r]) (void)hipEventDestroy(ctx->ev_arr[r]);
    }
    delete ctx;
}

}  // extern "C"
