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
//                                    reductions); dz is then handed to the matrix cores
//   W[o][k] -= eta dz_o x[k];  U[o][k] += dz_o x[k]      in registers, as 4 x 4 outer products
//                                    on the matrix cores (g never stored)
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

// ---- the round kernel: rank-1 updates on the matrix cores ----------------------------------
// Two thirds of a recursion's multiply-adds are the rank-1 updates  W -= eta dz x^T  and
// U += dz x^T.  v_mfma_f32_4x4x1_16b_f32 computes 16 independent 4 x 4 outer products
// D[b] += A[b] B[b]^T: lane l supplies A[b = l/4][i = l%4] and B[b][n = l%4] and receives, in
// its four result registers, the products of the four A entries of its block with ITS OWN B
// entry.  With B = the lane's own column of the sampled row and A = four entries of
// (-eta) dz (the same four in every block), one instruction updates four class rows of the
// lane's own column: the replica keeps the ownership it has in the vector-ALU form (thread t
// owns columns t, t+512, ... of every class row), so the logits still need no other lane's
// data, and three instructions per 64 columns cover classes 0..11 (rows 10 and 11 stay
// zero).  The vector ALU is left with the dot products, the reductions and the softmax.
// NC columns per thread; EXACT: D == 512 * NC, no column guards.
typedef float f4v __attribute__((ext_vector_type(4)));

template <int NC, bool EXACT>
__global__ void __launch_bounds__(kSmThreads, 1)
k_softmax_round(const RoundParams *__restrict__ rp, const float *Wg, int D) {
    constexpr int C = 10, Q = 3;   // classes, groups of four class rows
    const RoundParams p = rp[blockIdx.x];
    const gcf_ptr Xg = as_global(p.X);
    const gci_ptr yg = as_global(p.y);
    const gf_ptr Wc = as_global(p.W), Uc = as_global(p.U);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, cls = lane & 15;

    __shared__ float zpart[2][kSmWaves][16];

    if (!Wg) Wg = p.W;
    f4v W[NC][Q], U[NC][Q];
#pragma unroll
    for (int j = 0; j < NC; ++j) {
        const int k = tid + kSmThreads * j;
#pragma unroll
        for (int q = 0; q < Q; ++q)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int o = 4 * q + r;
                W[j][q][r] = (o < C && (EXACT || k < D)) ? Wg[(int64_t)o * D + k] : 0.f;
                U[j][q][r] = 0.f;
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

    auto recursion = [&](int u, const float (&x)[NC], int lab, float (&xn)[NC], int &labn) {
        // prefetch (Algorithm 2, sampling step; the index is a counter hash)
        if (u + 1 < p.m) load_row(sample_row(p.key, (uint64_t)(p.q0 + u + 1), p.n_samples), xn, labn);
        float(*zp)[16] = zpart[u & 1];
        float s[C];
#pragma unroll
        for (int o = 0; o < C; ++o) {
            s[o] = 0.f;
#pragma unroll
            for (int j = 0; j < NC; ++j) s[o] += W[j][o >> 2][o & 3] * x[j];
        }
        float t[(C + 3) / 4];
        wave_sum_rows<C>(s, t);
        if (cls == 0) {
            const int row = lane >> 4, o0 = ((row & 1) << 1) | (row >> 1);
#pragma unroll
            for (int k = 0; k < (C + 3) / 4; ++k)
                if (4 * k + o0 < C) zp[wave][4 * k + o0] = t[k];
        }
        __syncthreads();
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
        // w <- w - eta g, U <- U + g with g = dz x^T: lane l hands the matrix core entry
        // 4q + l%4 of dz (lanes 10..15 of a row hold zeros) and its own x
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const float a = __shfl(dzl, 4 * q + (lane & 3), 64);
            const float na = -p.eta * a;
#pragma unroll
            for (int j = 0; j < NC; ++j) {
                W[j][q] = __builtin_amdgcn_mfma_f32_4x4x1f32(na, x[j], W[j][q], 0, 0, 0);
                U[j][q] = __builtin_amdgcn_mfma_f32_4x4x1f32(a, x[j], U[j][q], 0, 0, 0);
            }
        }
    };

    float xa[NC], xb[NC];
    int la = 0, lb = 0;
    if (p.m > 0) load_row(sample_row(p.key, (uint64_t)p.q0, p.n_samples), xa, la);
    int u = 0;
    for (; u + 1 < p.m; u += 2) {
        recursion(u, xa, la, xb, lb);
        recursion(u + 1, xb, lb, xa, la);
    }
    if (u < p.m) recursion(u, xa, la, xb, lb);

#pragma unroll
    for (int j = 0; j < NC; ++j) {
        const int k = tid + kSmThreads * j;
        if (EXACT || k < D) {
#pragma unroll
            for (int o = 0; o < C; ++o) {
                Wc[(int64_t)o * D + k] = W[j][o >> 2][o & 3];
                Uc[(int64_t)o * D + k] = U[j][o >> 2][o & 3];
            }
        }
    }
    if (tid < C) {
        Wc[(int64_t)C * D + tid] = bias;
        Uc[(int64_t)C * D + tid] = Ub;
    }
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
        k_softmax_round<1, false><<<nact, kSmThreads, 0, s>>>(dp, Wg, D);
    else if (D <= 2 * kSmThreads)
        k_softmax_round<2, false><<<nact, kSmThreads, 0, s>>>(dp, Wg, D);
    else if (D == 6 * kSmThreads)
        k_softmax_round<6, true><<<nact, kSmThreads, 0, s>>>(dp, Wg, D);
    else
        k_softmax_round<6, false><<<nact, kSmThreads, 0, s>>>(dp, Wg, D);
    if (timed) prof->after(F_SOFTMAX_ROUND, s);
    return hipGetLastError();
}

}  // namespace aet
