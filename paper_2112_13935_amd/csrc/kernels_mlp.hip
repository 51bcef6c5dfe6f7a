// Fused local round for dense-ReLU-dense models (D -> H -> C, mini-batch B = 16 or 32).
//
// One launch runs the whole round (Algorithm 2, MainComputeNode: all s_i/B recursions) of
// every active client.  A client is handled by a cluster of G = H/16 workgroups; workgroup
// g owns hidden units 16g..16g+15: its slice of the first layer (16 x D weights, 16
// biases) and of the second layer (C x 16 weights), together with the matching slices of
// U, stay in registers / LDS for the whole round, so the per-recursion traffic is the
// mini-batch rows plus one small exchange:
//
//   per recursion: gather the B rows into LDS; z1 = X W1^T on the matrix cores (fp32 MFMA
//   16x16x4; the K range is split over the 4 waves and summed through LDS); h = relu(z1 +
//   b1); partial logits of the 16 own units -> a 16-float-per-sample record in global
//   memory; cluster barrier; every workgroup sums the G records, softmax, d logits;
//   dh = (W2^T d logits) * 1[h > 0]; dW1^T = X^T dh again on the matrix cores, whose
//   accumulator tile has exactly the register layout the forward pass needs as its B
//   operand, so  w <- w - eta g  and  U <- U + g  are applied to registers in place.
//
// The cluster barrier is a counter in global memory (release/acquire at agent scope) and
// needs all G workgroups of a client resident at once: the launcher never launches more
// workgroups than the device can hold (1 per compute unit with this LDS footprint).  The
// wait is bounded: on expiry an error flag is raised and every workgroup still runs to
// the end, so the grid always drains.
#include "aet_device.h"
#include "aet_internal.h"

namespace aet {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kMlpTPW = 13;          // K tiles (of 16) per wave  => D <= 16*4*13 = 832
constexpr int kMlpMaxG = 16;         // workgroups per client
constexpr int kSpinLimit = 1 << 22;  // bounded wait of the cluster barrier

__device__ __forceinline__ void store_agent(float *p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_agent(const float *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// All threads of the workgroup call this.  Returns after every workgroup of the cluster
// has arrived `target` times in total (or the wait expired and the error flag is set).
__device__ __forceinline__ void cluster_barrier(int *counter, int target, int *errflag) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __syncthreads();
    if (threadIdx.x == 0) {
        __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int spins = 0;
        while (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            __builtin_amdgcn_s_sleep(1);
            if ((++spins & 1023) == 0) {
                if (spins >= kSpinLimit ||
                    __hip_atomic_load(errflag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                    __hip_atomic_store(errflag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
            }
        }
    }
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

template <int NBT>
__global__ void __launch_bounds__(256, 1)
k_mlp_round(const RoundParams *__restrict__ rp, int a0, int nact, const float *__restrict__ Wg,
            int D, int H, int C, int G, float *__restrict__ xbuf, int *__restrict__ counters,
            int *__restrict__ errflag) {
    constexpr int B = 16 * NBT;
    // workgroup -> (client, unit group): consecutive workgroup ids go round the 8 XCDs, so
    // the G workgroups of one client are given ids that land on the same XCD and share
    // its L2 for the mini-batch rows.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int a = a0 + xcd + 8 * (slot / G);
    const int g = slot % G;
    if (a >= nact) return;
    const RoundParams p = rp[a];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 15, lg = lane >> 4;
    const int KT = (D + 15) >> 4;
    const int ld = KT * 16 + 4;

    extern __shared__ float smem[];
    float *Xs = smem;                 // [B][ld]
    float *red = Xs + B * ld;         // [4][B][16]
    float *hs = red + 4 * B * 16;     // [B][16]
    float *dhs = hs + B * 16;         // [B][16]
    float *zs = dhs + B * 16;         // [B][16]  logits, then d logits
    float *W2s = zs + B * 16;         // [16][16] (o, j)
    float *U2s = W2s + 256;
    float *b1s = U2s + 256;           // [16]
    float *Ub1s = b1s + 16;
    float *b2s = Ub1s + 16;
    float *Ub2s = b2s + 16;
    float *lossb = Ub2s + 16;         // [B]
    int *rows = reinterpret_cast<int *>(lossb + B);
    int *labs = rows + B;

    const int64_t b1_off = (int64_t)H * D, w2_off = b1_off + H, b2_off = w2_off + (int64_t)C * H;
    const float invB = 1.0f / (float)B;

    // ---- adopt the global model: own slice into registers / LDS; U = 0 -----------------
    f4 W1r[kMlpTPW], U1r[kMlpTPW];
#pragma unroll
    for (int tt = 0; tt < kMlpTPW; ++tt) {
        const int t = tt * 4 + wave;
        f4 w = {0.f, 0.f, 0.f, 0.f};
        if (t < KT) {
            const float *src = Wg + (int64_t)(16 * g + li) * D;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int k = 16 * t + 4 * lg + r;
                if (k < D) w[r] = src[k];
            }
        }
        W1r[tt] = w;
        U1r[tt] = f4{0.f, 0.f, 0.f, 0.f};
    }
    {
        const int o = tid >> 4, j = tid & 15;  // 256 threads = 16 x 16
        W2s[tid] = (o < C) ? Wg[w2_off + (int64_t)o * H + 16 * g + j] : 0.f;
        U2s[tid] = 0.f;
        if (tid < 16) {
            b1s[tid] = Wg[b1_off + 16 * g + tid];
            Ub1s[tid] = 0.f;
            b2s[tid] = (tid < C) ? Wg[b2_off + tid] : 0.f;
            Ub2s[tid] = 0.f;
        }
    }
    float loss_acc = 0.f;
    int *counter = counters + a;
    __syncthreads();

    for (int u = 0; u < p.m; ++u) {
        // ---- sample indices of the mini-batch (Algorithm 2: sample xi from D_c) ---------
        if (tid < B) {
            const uint32_t row = sample_row(p.key, (uint64_t)(p.q0 + (int64_t)u * B + tid), p.n_samples);
            rows[tid] = (int)row;
            labs[tid] = p.y[row];
        }
        __syncthreads();
        // ---- gather the rows into LDS (pad columns to a multiple of 16 with zeros) ------
        {
            const int vec_per_row = KT * 4;  // float4 per padded row
            for (int i = tid; i < B * vec_per_row; i += 256) {
                const int b = i / vec_per_row, v = i - b * vec_per_row;
                const float *src = p.X + (int64_t)rows[b] * D + 4 * v;
                f4 x;
                if (4 * v + 3 < D && (D & 3) == 0) {
                    x = *reinterpret_cast<const f4 *>(src);
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) x[r] = (4 * v + r < D) ? src[r] : 0.f;
                }
                *reinterpret_cast<f4 *>(Xs + b * ld + 4 * v) = x;
            }
        }
        __syncthreads();
        // ---- z1 partial sums on the matrix cores ----------------------------------------
        {
            f4 acc[NBT];
#pragma unroll
            for (int bt = 0; bt < NBT; ++bt) acc[bt] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int tt = 0; tt < kMlpTPW; ++tt) {
                const int t = tt * 4 + wave;
                if (t < KT) {
#pragma unroll
                    for (int bt = 0; bt < NBT; ++bt) {
                        const f4 x = *reinterpret_cast<const f4 *>(Xs + (16 * bt + li) * ld + 16 * t + 4 * lg);
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            acc[bt] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[r], W1r[tt][r], acc[bt], 0, 0, 0);
                    }
                }
            }
#pragma unroll
            for (int bt = 0; bt < NBT; ++bt)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    red[(wave * B + 16 * bt + 4 * lg + r) * 16 + li] = acc[bt][r];
        }
        __syncthreads();
        // ---- h = relu(z1 + b1) ----------------------------------------------------------
        for (int i = tid; i < B * 16; i += 256) {
            float s = b1s[i & 15] + red[i] + red[B * 16 + i] + red[2 * B * 16 + i] + red[3 * B * 16 + i];
            hs[i] = s > 0.f ? s : 0.f;
        }
        __syncthreads();
        // ---- partial logits of the own 16 units -> exchange record ----------------------
        float *rec = xbuf + ((int64_t)(a * 2 + (u & 1)) * kMlpMaxG) * (B * 16);
        for (int i = tid; i < B * 16; i += 256) {
            const int b = i >> 4, o = i & 15;
            float s = 0.f;
            if (o < C) {
#pragma unroll
                for (int j = 0; j < 16; ++j) s += W2s[o * 16 + j] * hs[b * 16 + j];
            }
            store_agent(rec + (int64_t)g * (B * 16) + i, s);
        }
        cluster_barrier(counter, G * (u + 1), errflag);
        for (int i = tid; i < B * 16; i += 256) {
            float s = b2s[i & 15];
            for (int gg = 0; gg < G; ++gg) s += load_agent(rec + (int64_t)gg * (B * 16) + i);
            zs[i] = s;
        }
        __syncthreads();
        // ---- softmax cross-entropy, d logits --------------------------------------------
        if (tid < B) {
            float *z = zs + tid * 16;
            const int lab = labs[tid];
            float zmax = z[0];
            for (int j = 1; j < C; ++j) zmax = fmaxf(zmax, z[j]);
            float sum = 0.f;
            for (int j = 0; j < C; ++j) sum += expf(z[j] - zmax);
            const float lse = zmax + logf(sum);
            lossb[tid] = lse - z[lab];
            for (int j = 0; j < 16; ++j) z[j] = (j < C) ? expf(z[j] - lse) - (j == lab ? 1.f : 0.f) : 0.f;
        }
        __syncthreads();
        if (g == 0 && tid == 0) {
            float s = 0.f;
            for (int b = 0; b < B; ++b) s += lossb[b];
            loss_acc += s * invB;
        }
        // ---- dh = (W2^T dz) * 1[h > 0] --------------------------------------------------
        for (int i = tid; i < B * 16; i += 256) {
            const int b = i >> 4, j = i & 15;
            float s = 0.f;
            for (int o = 0; o < C; ++o) s += W2s[o * 16 + j] * zs[b * 16 + o];
            dhs[i] = hs[i] > 0.f ? s : 0.f;
        }
        __syncthreads();
        // ---- second layer and biases: g, then w -= eta g, U += g ------------------------
        {
            const int o = tid >> 4, j = tid & 15;
            if (o < C) {
                float s = 0.f;
                for (int b = 0; b < B; ++b) s += zs[b * 16 + o] * hs[b * 16 + j];
                s *= invB;
                W2s[tid] -= p.eta * s;
                U2s[tid] += s;
            }
            if (tid < 16) {
                float s = 0.f;
                for (int b = 0; b < B; ++b) s += dhs[b * 16 + tid];
                s *= invB;
                b1s[tid] -= p.eta * s;
                Ub1s[tid] += s;
            } else if (tid < 32 && tid - 16 < C) {
                const int oo = tid - 16;
                float s = 0.f;
                for (int b = 0; b < B; ++b) s += zs[b * 16 + oo];
                s *= invB;
                b2s[oo] -= p.eta * s;
                Ub2s[oo] += s;
            }
        }
        // ---- first layer: dW1^T = X^T dh on the matrix cores, update in registers -------
        {
            float dhb[4 * NBT];
#pragma unroll
            for (int s = 0; s < 4 * NBT; ++s) dhb[s] = dhs[(4 * s + lg) * 16 + li];
            const float eb = p.eta * invB;
#pragma unroll
            for (int tt = 0; tt < kMlpTPW; ++tt) {
                const int t = tt * 4 + wave;
                if (t < KT) {
                    f4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int s = 0; s < 4 * NBT; ++s)
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(Xs[(4 * s + lg) * ld + 16 * t + li], dhb[s], acc, 0, 0, 0);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        W1r[tt][r] -= eb * acc[r];
                        U1r[tt][r] += invB * acc[r];
                    }
                }
            }
        }
        __syncthreads();
    }

    // ---- end of round: the replica and the message payload go to HBM ---------------------
#pragma unroll
    for (int tt = 0; tt < kMlpTPW; ++tt) {
        const int t = tt * 4 + wave;
        if (t < KT) {
            const int64_t base = (int64_t)(16 * g + li) * D;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int k = 16 * t + 4 * lg + r;
                if (k < D) {
                    p.W[base + k] = W1r[tt][r];
                    p.U[base + k] = U1r[tt][r];
                }
            }
        }
    }
    {
        const int o = tid >> 4, j = tid & 15;
        if (o < C) {
            p.W[w2_off + (int64_t)o * H + 16 * g + j] = W2s[tid];
            p.U[w2_off + (int64_t)o * H + 16 * g + j] = U2s[tid];
        }
        if (tid < 16) {
            p.W[b1_off + 16 * g + tid] = b1s[tid];
            p.U[b1_off + 16 * g + tid] = Ub1s[tid];
            if (g == 0 && tid < C) {
                p.W[b2_off + tid] = b2s[tid];
                p.U[b2_off + tid] = Ub2s[tid];
            }
        }
        if (g == 0 && tid == 0) *p.loss = loss_acc;
    }
}

__global__ void k_zero_ints(int *p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

static size_t mlp_lds_bytes(int D, int B) {
    const int KT = (D + 15) / 16, ld = KT * 16 + 4;
    return sizeof(float) * ((size_t)B * ld + 4 * B * 16 + 3 * B * 16 + 512 + 64 + B) + sizeof(int) * 2 * B;
}

bool mlp_round_supported(int D, int H, int C, int B) {
    if (!(B == 16 || B == 32)) return false;
    if (H % 16 || H / 16 > kMlpMaxG || C < 1 || C > 16) return false;
    if (D < 1 || (D + 15) / 16 > 4 * kMlpTPW) return false;
    return mlp_lds_bytes(D, B) <= 160 * 1024;
}

size_t mlp_round_scratch_bytes(int n_clients, int B) {
    // exchange records [client][2][kMlpMaxG][B*16] floats, one counter per client, one flag
    return (size_t)n_clients * 2 * kMlpMaxG * B * 16 * 4 + ((size_t)n_clients + 64) * 4;
}

static int g_mlp_capacity[2] = {0, 0};  // resident workgroups per device, per NBT

template <int NBT>
static hipError_t mlp_capacity(size_t lds, int *cap) {
    if (g_mlp_capacity[NBT - 1] > 0) { *cap = g_mlp_capacity[NBT - 1]; return hipSuccess; }
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_mlp_round<NBT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    int dev = 0, cus = 0, per_cu = 0;
    e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_mlp_round<NBT>, 256, lds);
    if (e != hipSuccess) return e;
    *cap = cus * per_cu;
    return hipSuccess;
}

template <int NBT>
static hipError_t mlp_launch(hipStream_t s, Profiler *prof, const RoundParams *dp, int nact, const float *Wg,
                             int D, int H, int C, void *scratch, int n_clients) {
    constexpr int B = 16 * NBT;
    const int G = H / 16;
    const size_t lds = mlp_lds_bytes(D, B);
    int cap = 0;
    hipError_t e = mlp_capacity<NBT>(lds, &cap);
    if (e != hipSuccess) return e;
    // Clusters per launch: every workgroup that waits in the cluster barrier must be
    // resident together with its peers.  Workgroups of unused slots exit at once and free
    // their compute unit, so only the working ones count.
    const int per_launch = cap / G;
    if (per_launch < 1) return hipErrorLaunchOutOfResources;
    float *xbuf = static_cast<float *>(scratch);
    int *counters = reinterpret_cast<int *>(xbuf + (size_t)n_clients * 2 * kMlpMaxG * B * 16);
    int *errflag = counters + n_clients;
    k_zero_ints<<<(nact + 255) / 256, 256, 0, s>>>(counters, nact);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    for (int a0 = 0; a0 < nact; a0 += per_launch) {
        const int here = (nact - a0 < per_launch) ? nact - a0 : per_launch;
        const int groups = (here + 7) / 8;  // clients per XCD in this launch
        const unsigned grid = (unsigned)(8 * groups * G);
        if (prof && prof->on[F_MLP_ROUND]) prof->before(F_MLP_ROUND, s);
        k_mlp_round<NBT><<<grid, 256, lds, s>>>(dp, a0, (a0 + here), Wg, D, H, C, G, xbuf, counters, errflag);
        if (prof && prof->on[F_MLP_ROUND]) prof->after(F_MLP_ROUND, s);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_mlp_round(hipStream_t s, Profiler *prof, const RoundParams *dp, int nact,
                            const float *Wg, int D, int H, int C, int B, void *scratch,
                            int n_clients) {
    if (nact <= 0) return hipSuccess;
    return B == 16 ? mlp_launch<1>(s, prof, dp, nact, Wg, D, H, C, scratch, n_clients)
                   : mlp_launch<2>(s, prof, dp, nact, Wg, D, H, C, scratch, n_clients);
}

hipError_t mlp_clear_error_flag(hipStream_t s, void *scratch, int n_clients, int B) {
    float *xbuf = static_cast<float *>(scratch);
    int *counters = reinterpret_cast<int *>(xbuf + (size_t)n_clients * 2 * kMlpMaxG * B * 16);
    k_zero_ints<<<1, 64, 0, s>>>(counters + n_clients, 1);
    return hipGetLastError();
}

const int *mlp_error_flag_ptr(void *scratch, int n_clients, int B) {
    float *xbuf = static_cast<float *>(scratch);
    int *counters = reinterpret_cast<int *>(xbuf + (size_t)n_clients * 2 * kMlpMaxG * B * 16);
    return counters + n_clients;
}

}  // namespace aet
