// Fused local round for softmax regression (one dense layer D -> C, per-sample SGD, B = 1).
//
// One workgroup (8 waves) per client runs the client's whole round (Algorithm 2,
// MainComputeNode: s_i recursions).  The replica w_c (C x D weights + C biases) and the
// gradient sum U stay in registers for the round: thread t owns columns t, t+512, ... of
// every class row.  Per recursion the only memory traffic is the sampled row (prefetched one
// recursion ahead: the index hash is a counter, so the next row is known) and its label.
//
//   z_o = b_o + sum_k W[o][k] x[k]   per-thread partial sums, DPP reduction inside a wave,
//                                    one LDS hop across the 8 waves (fixed order)
//   p = softmax(z), dz = p - onehot  lane o of every 16-lane row handles class o (DPP row
//                                    reductions); dz is then read lane by lane
//   W[o][k] -= eta dz_o x[k];  U[o][k] += dz_o x[k]      in registers (g never stored)
//
// At the end of the round w_c and U are written to HBM once.
#include "aet_device.h"
#include "aet_internal.h"

namespace aet {

constexpr int kSmThreads = 512;
constexpr int kSmWaves = kSmThreads / 64;

// sum over the 64 lanes of a wave; the total ends up in lane 63
__device__ __forceinline__ float wave_sum_dpp(float v) {
    // within quads, then across the halves of 8 and 16 lanes of a row
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));
    // lane 15 of a row to the next row (rows 1 and 3), then lane 31 to rows 2 and 3
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x142, 0xA, 0xF, false));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x143, 0xC, 0xF, false));
    return v;
}

#define AET_DPP_ADD(v, ctrl, rmask, bc) \
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), ctrl, rmask, 0xF, bc))
template <int N>
__device__ __forceinline__ void wave_sum_dpp_many(float (&v)[N]) {
#pragma unroll
    for (int o = 0; o < N; ++o) AET_DPP_ADD(v[o], 0xB1, 0xF, true);
#pragma unroll
    for (int o = 0; o < N; ++o) AET_DPP_ADD(v[o], 0x4E, 0xF, true);
#pragma unroll
    for (int o = 0; o < N; ++o) AET_DPP_ADD(v[o], 0x141, 0xF, true);
#pragma unroll
    for (int o = 0; o < N; ++o) AET_DPP_ADD(v[o], 0x140, 0xF, true);
#pragma unroll
    for (int o = 0; o < N; ++o) AET_DPP_ADD(v[o], 0x142, 0xA, false);
#pragma unroll
    for (int o = 0; o < N; ++o) AET_DPP_ADD(v[o], 0x143, 0xC, false);
}
#undef AET_DPP_ADD

// Sums of N values over the 64 lanes of a wave, several values per instruction.  The lane
// swaps of gfx950 exchange half-waves (rows of 16 lanes) between two registers, so that one
// addition folds two (then four) different values at once:
//   swap32(a, b) -> [a.lo, b.lo], [a.hi, b.hi]; their sum holds a folded to 32 lanes in the
//                   lower half and b in the upper half;
//   swap16(p, q) -> rows [p0, q0, p2, q2], [p1, q1, p3, q3]; their sum holds four values, one
//                   per row of 16 lanes;
// four shuffle-and-add stages inside the rows finish.  Register k of the result holds, in all
// 16 lanes of row r, the total of value 4k + rowmap(r), rowmap = {0, 2, 1, 3}.
template <int N>
__device__ __forceinline__ void wave_sum_rows(const float (&v)[N], float (&out)[(N + 3) / 4]) {
    static_assert(N % 2 == 0, "values come in pairs");
    constexpr int NP = N / 2, NQ = (N + 3) / 4;
    float p[NP];
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const auto r = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(int, v[2 * k]),
                                                        __builtin_bit_cast(int, v[2 * k + 1]), false, false);
        p[k] = __builtin_bit_cast(float, (int)r[0]) + __builtin_bit_cast(float, (int)r[1]);
    }
#pragma unroll
    for (int k = 0; k < NQ; ++k) {
        const float a = p[2 * k], b = 2 * k + 1 < NP ? p[2 * k + 1] : 0.f;
        const auto r = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(int, a), __builtin_bit_cast(int, b), false, false);
        out[k] = __builtin_bit_cast(float, (int)r[0]) + __builtin_bit_cast(float, (int)r[1]);
    }
#pragma unroll
    for (int k = 0; k < NQ; ++k) out[k] += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, out[k]), 0xB1, 0xF, 0xF, true));
#pragma unroll
    for (int k = 0; k < NQ; ++k) out[k] += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, out[k]), 0x4E, 0xF, 0xF, true));
#pragma unroll
    for (int k = 0; k < NQ; ++k) out[k] += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, out[k]), 0x141, 0xF, 0xF, true));
#pragma unroll
    for (int k = 0; k < NQ; ++k) out[k] += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, out[k]), 0x140, 0xF, 0xF, true));
}

// sum / max over each row of 16 lanes (every lane of the row gets the result)
__device__ __forceinline__ float row_sum_dpp(float v) {
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));
    return v;
}
__device__ __forceinline__ float row_max_dpp(float v) {
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true)));
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true)));
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true)));
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true)));
    return v;
}

// C classes (<= 16), NC columns per thread; EXACT: D == 512 * NC, no column guards
template <int C, int NC, bool EXACT>
__global__ void __launch_bounds__(kSmThreads, 1)
k_softmax_round(const RoundParams *__restrict__ rp, const float *Wg, int D) {
    const RoundParams p = rp[blockIdx.x];
    const gcf_ptr Xg = as_global(p.X);
    const gci_ptr yg = as_global(p.y);
    const gf_ptr Wc = as_global(p.W), Uc = as_global(p.U);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, cls = lane & 15;

    __shared__ float zpart[2][kSmWaves][16];

    // adopt the global model (server form) or go on from the own replica (Wg == NULL:
    // peer-to-peer form); U = 0.  Lane `cls` of every row keeps bias and its U entry.
    if (!Wg) Wg = p.W;
    float W[C][NC], U[C][NC];
#pragma unroll
    for (int o = 0; o < C; ++o) {
#pragma unroll
        for (int j = 0; j < NC; ++j) {
            const int k = tid + kSmThreads * j;
            W[o][j] = (EXACT || k < D) ? Wg[(int64_t)o * D + k] : 0.f;
            U[o][j] = 0.f;
        }
    }
    float bias = cls < C ? Wg[(int64_t)C * D + cls] : 0.f, Ub = 0.f;
    float loss_acc = 0.f;

    auto load_row = [&](uint32_t row, float (&x)[NC], int &lab) {
#pragma unroll
        for (int j = 0; j < NC; ++j) {
            const int k = tid + kSmThreads * j;
            x[j] = (EXACT || k < D) ? Xg[(int64_t)row * D + k] : 0.f;
        }
        lab = yg[row];
    };

    // one recursion on sample x; meanwhile the next sample is fetched into xn
    auto recursion = [&](int u, const float (&x)[NC], int lab, float (&xn)[NC], int &labn) {
        // prefetch (Algorithm 2, sampling step; the index is a counter hash)
        if (u + 1 < p.m) load_row(sample_row(p.key, (uint64_t)(p.q0 + u + 1), p.n_samples), xn, labn);
        // partial logits of this thread's columns, summed over the wave
        float(*zp)[16] = zpart[u & 1];
        float s[C];
#pragma unroll
        for (int o = 0; o < C; ++o) {
            s[o] = 0.f;
#pragma unroll
            for (int j = 0; j < NC; ++j) s[o] += W[o][j] * x[j];
        }
        // the C sums over the wave, four classes per register at the end; the first lane of
        // every row posts its classes
        float t[(C + 3) / 4];
        wave_sum_rows<C>(s, t);
        if (cls == 0) {
            const int row = lane >> 4, o0 = ((row & 1) << 1) | (row >> 1);
#pragma unroll
            for (int k = 0; k < (C + 3) / 4; ++k)
                if (4 * k + o0 < C) zp[wave][4 * k + o0] = t[k];
        }
        __syncthreads();
        // lane cls of every row: logit of class cls, then the softmax inside the row
        float z = bias;
#pragma unroll
        for (int w = 0; w < kSmWaves; ++w) z += zp[w][cls];
        const bool live = cls < C;
        const float zmax = row_max_dpp(live ? z : -3.0e38f);
        const float ex = live ? __expf(z - zmax) : 0.f;
        const float lse = zmax + __logf(row_sum_dpp(ex));
        const float dzl = live ? __expf(z - lse) - (cls == lab ? 1.f : 0.f) : 0.f;
        if (cls == lab) loss_acc += lse - z;
        bias -= p.eta * dzl;
        Ub += dzl;
        // w <- w - eta g, U <- U + g, with g = dz x^T; dz is read from the lanes that hold it
#pragma unroll
        for (int o = 0; o < C; ++o) {
            const float dz = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, dzl), o));
            const float ed = p.eta * dz;
#pragma unroll
            for (int j = 0; j < NC; ++j) {
                W[o][j] -= ed * x[j];
                U[o][j] += dz * x[j];
            }
        }
    };

    // two register sets alternate as "current" and "next" sample
    float xa[NC], xb[NC];
    int la = 0, lb = 0;
    if (p.m > 0) load_row(sample_row(p.key, (uint64_t)p.q0, p.n_samples), xa, la);
    int u = 0;
    for (; u + 1 < p.m; u += 2) {
        recursion(u, xa, la, xb, lb);
        recursion(u + 1, xb, lb, xa, la);
    }
    if (u < p.m) recursion(u, xa, la, xb, lb);

    // the replica and the message payload go to HBM
#pragma unroll
    for (int o = 0; o < C; ++o) {
#pragma unroll
        for (int j = 0; j < NC; ++j) {
            const int k = tid + kSmThreads * j;
            if (EXACT || k < D) {
                Wc[(int64_t)o * D + k] = W[o][j];
                Uc[(int64_t)o * D + k] = U[o][j];
            }
        }
    }
    if (tid < C) {
        Wc[(int64_t)C * D + tid] = bias;
        Uc[(int64_t)C * D + tid] = Ub;
    }
    // every thread with cls == label added the sample's loss: take wave 0, row 0
    if (wave == 0) {
        float l = lane < 16 ? loss_acc : 0.f;
        l = wave_sum_dpp(l);
        if (lane == 63) *as_global(p.loss) = l;
    }
}

bool softmax_round_supported(int D, int C, int B) {
    return B == 1 && C == 10 && D >= 1 && D <= kSmThreads * 6;
}

hipError_t launch_softmax_round(hipStream_t s, Profiler *prof, const RoundParams *dp, int nact,
                                const float *Wg, int D, int C) {
    if (nact <= 0) return hipSuccess;
    (void)C;
    const bool timed = prof && prof->on[F_SOFTMAX_ROUND];
    if (timed) prof->before(F_SOFTMAX_ROUND, s);
    if (D <= kSmThreads)
        k_softmax_round<10, 1, false><<<nact, kSmThreads, 0, s>>>(dp, Wg, D);
    else if (D <= 2 * kSmThreads)
        k_softmax_round<10, 2, false><<<nact, kSmThreads, 0, s>>>(dp, Wg, D);
    else if (D == 6 * kSmThreads)
        k_softmax_round<10, 6, true><<<nact, kSmThreads, 0, s>>>(dp, Wg, D);
    else
        k_softmax_round<10, 6, false><<<nact, kSmThreads, 0, s>>>(dp, Wg, D);
    if (timed) prof->after(F_SOFTMAX_ROUND, s);
    return hipGetLastError();
}

}  // namespace aet
