// Internal declarations shared by the host scheduler and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

namespace aet {

// Resolved geometry of one layer (activations are C,H,W per sample).
struct LayerGeom {
    int type, relu, k, pad;
    int ic, ih, iw, oc, oh, ow;
    int64_t w_off, b_off;       // offsets into the flat parameter vector
    int64_t in_size, out_size;  // floats per sample
};

// Everything a kernel needs to know about one client's round of this tick.
// One record per ACTIVE client; the array lives in device memory.
struct RoundParams {
    const float *X;      // shard rows
    const int32_t *y;    // shard labels
    float *W;            // the client's replica w_c (P floats)
    float *U;            // the slot that receives this round's gradient sum
    float *loss;         // accumulates the per-recursion mean loss
    uint64_t key;        // SplitMix64 stream key of (seed, client)
    int64_t q0;          // sample counter at the start of the round
    uint32_t n_samples;  // rows in the shard
    int32_t m;           // recursions in this round
    float eta;           // round step size
    int32_t client;
};

// One arriving message: w -= scale * U at the server, or at every neighbour of the sender.
struct Arrival {
    const float *U;
    float scale;
    int32_t sender;
};

// A short arrival list that is passed to the kernel by value.
constexpr int kArrivalPack = 32;
struct ArrivalPack {
    Arrival a[kArrivalPack];
};

// Device scratch of the layer-by-layer engine; all sized for n_clients * batch samples.
struct LayerScratch {
    float *act[17];     // act[0] = gathered inputs, act[l+1] = output of layer l
    float *del[17];     // d loss / d act[l] (l >= 1)
    uint8_t *amax[16];  // pool layers: which of the 4 window elements was the maximum
    int32_t *labels;    // [n_clients][batch]
    float *wgrad;       // partial sums of the convolution weight gradients
    bool plain;         // use the plain (non matrix-core) layer kernels
};

// Kernel families, for the optional per-launch timing with HIP events.
enum Family {
    F_BEGIN_ROUND = 0, F_GATHER, F_DENSE_FWD, F_DENSE_BWD_DATA, F_DENSE_BWD_WEIGHT, F_CONV_FWD,
    F_CONV_BWD_DATA, F_CONV_BWD_WEIGHT, F_POOL_FWD, F_POOL_BWD, F_SOFTMAX_CE, F_SERVER_REDUCE,
    F_SOFTMAX_ROUND, F_MLP_ROUND, F_NEIGHBOUR_APPLY, F_LENET_ROUND, F_COUNT
};
const char *family_name(int fam);

// Times the launches of the enabled families with event pairs recorded on the launch
// stream; durations are summed when the pairs are drained.
struct Profiler {
    struct Pair { int fam; hipEvent_t a, b; };
    bool on[F_COUNT] = {};
    bool any = false;
    double total_ms[F_COUNT] = {};
    int64_t launches[F_COUNT] = {};
    std::vector<hipEvent_t> pool;
    std::vector<Pair> pending;
    hipEvent_t cur = nullptr;
    hipError_t status = hipSuccess;

    void before(int fam, hipStream_t s);
    void after(int fam, hipStream_t s);
    hipError_t drain(hipStream_t s);
    void clear();
    ~Profiler();
};

// ---- launchers (each returns the launch status) --------------------------------------
// Wg == NULL (here and in the fused round kernels): the clients go on from their own replicas
hipError_t launch_begin_round(hipStream_t s, Profiler *prof, const RoundParams *dp, int nact,
                              const float *Wg, int64_t P);
hipError_t launch_layer_step(hipStream_t s, Profiler *prof, const RoundParams *dp, int nact, int u,
                             const LayerGeom *lay, int L, int B, const LayerScratch &sc);
hipError_t launch_server_reduce(hipStream_t s, Profiler *prof, float *Wg, const Arrival *darr,
                                int n_arr, int64_t P);
hipError_t launch_server_apply_small(hipStream_t s, Profiler *prof, float *Wg, const ArrivalPack &pack,
                                     int n_arr, int64_t P);
// Receive at the neighbours: replica r takes the arrivals whose sender is in nbr[nbr_off[r] ..
// nbr_off[r+1]), in list order.  The list comes by value (pack != NULL, n_arr <= kArrivalPack)
// or from device memory (darr).  W: the replicas, Ps floats apart.
hipError_t launch_apply_neighbour_U(hipStream_t s, Profiler *prof, float *W, int64_t Ps, int64_t P,
                                    int n_clients, const int32_t *nbr_off, const int32_t *nbr,
                                    const ArrivalPack *pack, const Arrival *darr, int n_arr);
// every replica (Ps floats apart, Ps a multiple of 4) <- src (Ps floats readable)
hipError_t launch_broadcast_model(hipStream_t s, float *W, int64_t Ps, int n_clients, const float *src);
hipError_t launch_debug_indices(hipStream_t s, uint64_t key, int64_t q0, int count,
                                uint32_t n_samples, int32_t *dst);
// convolution on the matrix cores (kernels_conv_mfma.hip); bwd = backward-data
bool conv_mfma_supported(const LayerGeom &L, bool bwd);
hipError_t launch_conv_mfma(hipStream_t s, Profiler *prof, const RoundParams *dp, int nact, int u, int B,
                            const LayerGeom &L, bool bwd, const float *src, float *dst,
                            const float *mask_src);
bool conv_wgrad_mfma_supported(const LayerGeom &L, int B);
size_t conv_wgrad_partial_floats(const LayerGeom &L, int B, int n_clients);
hipError_t launch_conv_wgrad_mfma(hipStream_t s, Profiler *prof, const RoundParams *dp, int nact, int u,
                                  int B, const LayerGeom &L, const float *in, const float *dout,
                                  float *partial);
// dense layers on the matrix cores (kernels_dense_mfma.hip); mode 0 fwd, 1 bwd-data, 2 bwd-weight
hipError_t launch_dense_mfma(hipStream_t s, Profiler *prof, int mode, const RoundParams *dp, int nact,
                             int u, int B, int K, int O, int64_t w_off, int64_t b_off, int relu,
                             const float *x, const float *y, float *z, const float *mask_src);
// fused round of softmax regression, per-sample SGD (kernels_softmax.hip)
bool softmax_round_supported(int D, int C, int B);
hipError_t launch_softmax_round(hipStream_t s, Profiler *prof, const RoundParams *dp, int nact,
                                const float *Wg, int D, int C);
// fused round of dense-ReLU-dense models (kernels_mlp.hip)
bool mlp_round_supported(int D, int H, int C, int B);
size_t mlp_round_scratch_bytes(int n_clients, int B);
// hp: HOST array of the tick's round records (they are passed on in kernel arguments)
hipError_t launch_mlp_round(hipStream_t s, Profiler *prof, const RoundParams *hp, int nact,
                            int max_m, const float *Wg, int D, int H, int C, int B, void *scratch,
                            int n_clients, uint32_t *epoch);
hipError_t mlp_clear_error_flag(hipStream_t s, void *scratch, int n_clients, int B);
const int *mlp_error_flag_ptr(void *scratch, int n_clients, int B);
// fused round of LeNet-5-style models (kernels_lenet.hip); dp: DEVICE array of round records
bool lenet_round_supported(const LayerGeom *lay, int L, int B);
size_t lenet_round_scratch_bytes(int n_clients);
hipError_t launch_lenet_round(hipStream_t s, Profiler *prof, const RoundParams *dp, int nact, int max_m,
                              const float *Wg, const LayerGeom *lay, int L, int B, void *scratch,
                              int n_clients, uint32_t *epoch);
hipError_t lenet_clear_error_flag(hipStream_t s, void *scratch, int n_clients);
const int *lenet_error_flag_ptr(void *scratch, int n_clients);

}  // namespace aet
