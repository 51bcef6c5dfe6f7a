// Server step (Algorithm 2, Receive, in its client-server form):
//   w_global <- w_global - sum over this tick's arrivals of (agg_scale * eta_k) * U_{k,c}.
// The U's are streamed once from HBM.  With few arrivals a single pass applies them in
// order; with many, the arrivals are cut into chunks that are summed in parallel
// (each chunk in order) and the chunk sums are then applied in order, so the result does
// not depend on how blocks are scheduled.
#include "aet_device.h"
#include "aet_internal.h"

namespace aet {

constexpr int kChunk = 16;  // arrivals per chunk of the two-stage form

__global__ void __launch_bounds__(256)
k_server_apply(float *__restrict__ Wg, const Arrival *__restrict__ arr, int n_arr, int64_t P) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= P) return;
    float w = Wg[i];
    for (int j = 0; j < n_arr; ++j) w -= arr[j].scale * arr[j].U[i];
    Wg[i] = w;
}

// the same with the arrival list in the kernel arguments (no staging copy)
__global__ void __launch_bounds__(256)
k_server_apply_small(float *__restrict__ Wg, ArrivalPack pack, int n_arr, int64_t P) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= P) return;
    float w = Wg[i];
    for (int j = 0; j < n_arr; ++j) w -= pack.a[j].scale * as_global(pack.a[j].U)[i];
    Wg[i] = w;
}

__global__ void __launch_bounds__(256)
k_server_partial(const Arrival *__restrict__ arr, int n_arr, int64_t P, int64_t stride,
                 float *__restrict__ partial) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= P) return;
    const int j0 = blockIdx.y * kChunk;
    const int j1 = min(j0 + kChunk, n_arr);
    float s = 0.f;
    for (int j = j0; j < j1; ++j) s += arr[j].scale * arr[j].U[i];
    partial[(int64_t)blockIdx.y * stride + i] = s;
}

__global__ void __launch_bounds__(256)
k_server_finish(float *__restrict__ Wg, const float *__restrict__ partial, int chunks, int64_t P,
                int64_t stride) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= P) return;
    float w = Wg[i];
    for (int c = 0; c < chunks; ++c) w -= partial[(int64_t)c * stride + i];
    Wg[i] = w;
}

hipError_t launch_server_apply_small(hipStream_t s, Profiler *prof, float *Wg, const ArrivalPack &pack,
                                     int n_arr, int64_t P) {
    if (n_arr <= 0) return hipSuccess;
    const bool timed = prof && prof->on[F_SERVER_REDUCE];
    if (timed) prof->before(F_SERVER_REDUCE, s);
    k_server_apply_small<<<(unsigned)((P + 255) / 256), 256, 0, s>>>(Wg, pack, n_arr, P);
    if (timed) prof->after(F_SERVER_REDUCE, s);
    return hipGetLastError();
}

int server_reduce_chunks(int n_arr, int64_t P) {
    (void)P;
    return n_arr <= 2 * kChunk ? 1 : (n_arr + kChunk - 1) / kChunk;
}

hipError_t launch_server_reduce(hipStream_t s, Profiler *prof, float *Wg, const Arrival *darr,
                                int n_arr, int64_t P, float *partial, int max_chunks) {
    if (n_arr <= 0) return hipSuccess;
    const bool timed = prof && prof->on[F_SERVER_REDUCE];
    if (timed) prof->before(F_SERVER_REDUCE, s);
    const unsigned gx = (unsigned)((P + 255) / 256);
    const int chunks = server_reduce_chunks(n_arr, P);
    if (chunks == 1 || chunks > max_chunks) {
        k_server_apply<<<gx, 256, 0, s>>>(Wg, darr, n_arr, P);
        if (timed) prof->after(F_SERVER_REDUCE, s);
        return hipGetLastError();
    }
    const int64_t stride = (P + 63) / 64 * 64;
    k_server_partial<<<dim3(gx, chunks), 256, 0, s>>>(darr, n_arr, P, stride, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    k_server_finish<<<gx, 256, 0, s>>>(Wg, partial, chunks, P, stride);
    if (timed) prof->after(F_SERVER_REDUCE, s);
    return hipGetLastError();
}

}  // namespace aet
