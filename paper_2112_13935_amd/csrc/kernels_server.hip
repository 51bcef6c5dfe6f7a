// Receive (Algorithm 2), at the server and at the neighbours.
// Server step (Receive in its client-server form):
//   w_global <- w_global - sum over this tick's arrivals of (agg_scale * eta_k) * U_{k,c}.
// The U's are streamed once from HBM.  With few arrivals every thread applies them in order
// to its own parameters; with many, a workgroup's thread groups each sum a contiguous part of
// the list in order and the group sums are added in group order, so the result does not
// depend on how blocks are scheduled.
#include "aet_device.h"
#include "aet_internal.h"

namespace aet {

constexpr int kFewArrivals = 32;  // up to here one thread walks the whole list

typedef float sf4 __attribute__((ext_vector_type(4)));
typedef const sf4 __attribute__((address_space(1))) *gcv4_ptr;

// Every kernel here moves float4s: the models and the U slots are padded to a multiple of
// 64 floats (nv = padded length / 4), the padding is carried along and never looked at.
__global__ void __launch_bounds__(256)
k_server_apply(float *__restrict__ Wg, const Arrival *__restrict__ arr, int n_arr, int64_t nv) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nv) return;
    sf4 w = reinterpret_cast<const sf4 *>(Wg)[i];
#pragma unroll 4
    for (int j = 0; j < n_arr; ++j) w -= arr[j].scale * reinterpret_cast<gcv4_ptr>(as_global(arr[j].U))[i];
    reinterpret_cast<sf4 *>(Wg)[i] = w;
}

// the same with the arrival list in the kernel arguments (no staging copy)
__global__ void __launch_bounds__(256)
k_server_apply_small(float *__restrict__ Wg, ArrivalPack pack, int n_arr, int64_t nv) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nv) return;
    sf4 w = reinterpret_cast<const sf4 *>(Wg)[i];
#pragma unroll 4
    for (int j = 0; j < n_arr; ++j) w -= pack.a[j].scale * reinterpret_cast<gcv4_ptr>(as_global(pack.a[j].U))[i];
    reinterpret_cast<sf4 *>(Wg)[i] = w;
}

// Many arrivals in one pass: a workgroup owns 16 float4 columns of the model; its 16 thread
// groups each sum a contiguous sixteenth of the arrival list in list order (8 loads in flight),
// the group sums are added in group order in LDS and subtracted from the model.  No partial
// sums in memory, no second kernel; the result does not depend on scheduling.
constexpr int kOneCols = 16;   // float4 columns per workgroup
constexpr int kOneGroups = 16; // arrival groups per workgroup
constexpr int kOneFlight = 8;  // loads in flight per thread

__global__ void __launch_bounds__(256)
k_server_reduce_one(float *__restrict__ Wg, const Arrival *__restrict__ arr, int n_arr, int64_t nv) {
    const int tid = threadIdx.x, c = tid & (kOneCols - 1), grp = tid / kOneCols;
    const int64_t i = (int64_t)blockIdx.x * kOneCols + c;
    const bool valid = i < nv;
    const int64_t ii = valid ? i : 0;
    const int per = (n_arr + kOneGroups - 1) / kOneGroups;
    const int j0 = grp * per, j1 = min(j0 + per, n_arr);
    sf4 s = {0.f, 0.f, 0.f, 0.f};
    for (int j = j0; j < j1; j += kOneFlight) {
        sf4 u[kOneFlight];
        float sc[kOneFlight];
#pragma unroll
        for (int q = 0; q < kOneFlight; ++q) {
            const bool in = j + q < j1;
            const Arrival a = arr[in ? j + q : j];
            sc[q] = in ? a.scale : 0.f;
            u[q] = reinterpret_cast<gcv4_ptr>(as_global(a.U))[ii];
        }
#pragma unroll
        for (int q = 0; q < kOneFlight; ++q)
            if (j + q < j1) s += sc[q] * u[q];
    }
    __shared__ sf4 red[kOneGroups][kOneCols];
    red[grp][c] = s;
    __syncthreads();
    if (grp == 0 && valid) {
        sf4 w = reinterpret_cast<const sf4 *>(Wg)[i];
        sf4 t = red[0][c];
#pragma unroll
        for (int g = 1; g < kOneGroups; ++g) t += red[g][c];
        reinterpret_cast<sf4 *>(Wg)[i] = w - t;
    }
}

hipError_t launch_server_apply_small(hipStream_t s, Profiler *prof, float *Wg, const ArrivalPack &pack,
                                     int n_arr, int64_t P) {
    if (n_arr <= 0) return hipSuccess;
    const bool timed = prof && prof->on[F_SERVER_REDUCE];
    if (timed) prof->before(F_SERVER_REDUCE, s);
    const int64_t nv = (P + 63) / 64 * 16;
    k_server_apply_small<<<(unsigned)((nv + 255) / 256), 256, 0, s>>>(Wg, pack, n_arr, nv);
    if (timed) prof->after(F_SERVER_REDUCE, s);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Receive at the neighbours (Algorithm 2 as printed): replica r applies, in list order,
// the arrivals whose sender is one of its neighbours:  w_r -= (scale * eta_k) * U_{k,v}.
// One block owns kNbElems consecutive parameters of one replica.  Its first wave picks the
// matching arrivals out of the tick's list (a window of kNbWin at a time, order kept by
// ballot + prefix count); then every thread carries its parameters through them.
// ---------------------------------------------------------------------------------------
constexpr int kNbWin = 256;     // arrivals examined per window
constexpr int kNbVec = 8;       // float4 per thread
constexpr int kNbBatch = 2;     // arrivals whose loads are in flight together
constexpr int kNbElems = 256 * 4 * kNbVec;

typedef float nf4 __attribute__((ext_vector_type(4)));

template <bool PACK>
__global__ void __launch_bounds__(256)
k_apply_neighbour_U(float *__restrict__ W, int64_t Ps, const int32_t *__restrict__ nbr_off,
                    const int32_t *__restrict__ nbr, ArrivalPack pack,
                    const Arrival *__restrict__ arr, int n_arr) {
    const int r = blockIdx.y;
    const int n0 = nbr_off[r], n1 = nbr_off[r + 1];
    if (n0 == n1) return;
    __shared__ const float *selU[kNbWin];
    __shared__ float selS[kNbWin];
    __shared__ int nsel;
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)blockIdx.x * kNbElems + 4 * tid;
    float *Wr = W + (int64_t)r * Ps;
    nf4 w[kNbVec];
    bool loaded = false;

    for (int j0 = 0; j0 < n_arr; j0 += kNbWin) {
        if (PACK) {
            // the short list sits in the kernel arguments: a uniform scan, one writer
            if (tid == 0) {
                int cnt = 0;
                for (int j = 0; j < n_arr; ++j) {
                    const int v = pack.a[j].sender;
                    bool hit = false;
                    for (int q = n0; q < n1; ++q) hit = hit || nbr[q] == v;
                    if (hit) { selU[cnt] = pack.a[j].U; selS[cnt] = pack.a[j].scale; ++cnt; }
                }
                nsel = cnt;
            }
        } else if (tid < 64) {
            int cnt = 0;
            const int jend = min(j0 + kNbWin, n_arr);
            for (int t = j0; t < jend; t += 64) {
                const int j = t + tid;
                bool hit = false;
                Arrival a = {nullptr, 0.f, -1};
                if (j < jend) {
                    a = arr[j];
                    for (int q = n0; q < n1; ++q) hit = hit || nbr[q] == a.sender;
                }
                const unsigned long long mask = __ballot(hit);
                if (hit) {
                    const int pos = cnt + __popcll(mask & ((1ull << tid) - 1ull));
                    selU[pos] = a.U;
                    selS[pos] = a.scale;
                }
                cnt += __popcll(mask);
            }
            if (tid == 0) nsel = cnt;
        }
        __syncthreads();
        const int ns = nsel;
        if (ns > 0) {
            if (!loaded) {
#pragma unroll
                for (int v = 0; v < kNbVec; ++v) {
                    const int64_t i = base + 1024 * v;
                    w[v] = i < Ps ? *reinterpret_cast<const nf4 *>(Wr + i) : nf4{0.f, 0.f, 0.f, 0.f};
                }
                loaded = true;
            }
            // a few arrivals at a time: their loads are in flight together (an element beyond
            // the model reads the first one instead and is never stored), then they are applied
            // in list order
            for (int s0 = 0; s0 < ns; s0 += kNbBatch) {
                nf4 u[kNbBatch][kNbVec];
                float sc[kNbBatch];
#pragma unroll
                for (int q = 0; q < kNbBatch; ++q) {
                    const int s = s0 + q < ns ? s0 + q : s0;
                    const float *U = selU[s];
                    sc[q] = s0 + q < ns ? selS[s] : 0.f;
#pragma unroll
                    for (int v = 0; v < kNbVec; ++v) {
                        const int64_t i = base + 1024 * v;
                        u[q][v] = *reinterpret_cast<const nf4 __attribute__((address_space(1))) *>(as_global(U) + (i < Ps ? i : 0));
                    }
                }
#pragma unroll
                for (int q = 0; q < kNbBatch; ++q)
                    if (s0 + q < ns) {
#pragma unroll
                        for (int v = 0; v < kNbVec; ++v) w[v] -= sc[q] * u[q][v];
                    }
            }
        }
        __syncthreads();
    }
    if (loaded) {
#pragma unroll
        for (int v = 0; v < kNbVec; ++v) {
            const int64_t i = base + 1024 * v;
            if (i < Ps) *reinterpret_cast<nf4 *>(Wr + i) = w[v];
        }
    }
}

hipError_t launch_apply_neighbour_U(hipStream_t s, Profiler *prof, float *W, int64_t Ps, int64_t P,
                                    int n_clients, const int32_t *nbr_off, const int32_t *nbr,
                                    const ArrivalPack *pack, const Arrival *darr, int n_arr) {
    (void)P;
    if (n_arr <= 0) return hipSuccess;
    const bool timed = prof && prof->on[F_NEIGHBOUR_APPLY];
    if (timed) prof->before(F_NEIGHBOUR_APPLY, s);
    dim3 grid((unsigned)((Ps + kNbElems - 1) / kNbElems), (unsigned)n_clients);
    if (pack) {
        k_apply_neighbour_U<true><<<grid, 256, 0, s>>>(W, Ps, nbr_off, nbr, *pack, nullptr, n_arr);
    } else {
        ArrivalPack none = {};
        k_apply_neighbour_U<false><<<grid, 256, 0, s>>>(W, Ps, nbr_off, nbr, none, darr, n_arr);
    }
    if (timed) prof->after(F_NEIGHBOUR_APPLY, s);
    return hipGetLastError();
}

// every replica <- src (Setup: all nodes start from the same model)
__global__ void __launch_bounds__(256)
k_broadcast_model(float *__restrict__ W, int64_t Ps, const float *__restrict__ src) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // float4 index
    if (4 * i >= Ps) return;
    reinterpret_cast<sf4 *>(W + (int64_t)blockIdx.y * Ps)[i] = reinterpret_cast<const sf4 *>(src)[i];
}

hipError_t launch_broadcast_model(hipStream_t s, float *W, int64_t Ps, int n_clients, const float *src) {
    dim3 grid((unsigned)((Ps / 4 + 255) / 256), (unsigned)n_clients);
    k_broadcast_model<<<grid, 256, 0, s>>>(W, Ps, src);
    return hipGetLastError();
}

hipError_t launch_server_reduce(hipStream_t s, Profiler *prof, float *Wg, const Arrival *darr,
                                int n_arr, int64_t P) {
    if (n_arr <= 0) return hipSuccess;
    const bool timed = prof && prof->on[F_SERVER_REDUCE];
    if (timed) prof->before(F_SERVER_REDUCE, s);
    const int64_t nv = (P + 63) / 64 * 16;   // float4s per padded model
    if (n_arr <= kFewArrivals)
        k_server_apply<<<(unsigned)((nv + 255) / 256), 256, 0, s>>>(Wg, darr, n_arr, nv);
    else
        k_server_reduce_one<<<(unsigned)((nv + kOneCols - 1) / kOneCols), 256, 0, s>>>(Wg, darr, n_arr, nv);
    if (timed) prof->after(F_SERVER_REDUCE, s);
    return hipGetLastError();
}

}  // namespace aet
