// Dense layers of the layer-by-layer engine on the matrix cores (fp32 MFMA 16x16x4):
// one 64 x 64 output tile per workgroup, operands staged through LDS in chunks of 32 along
// the contraction, batched over the active clients (blockIdx.z).
//
//   FWD         out[b][o] = relu?(bias[o] + sum_k in[b][k] W[o][k])      M = b, N = o, K = k
//   BWD_DATA    din[b][k] = mask * sum_o dout[b][o] W[o][k]              M = b, N = k, K = o
//   BWD_WEIGHT  g[o][k]  = (1/B) sum_b dout[b][o] in[b][k], then
//               W -= eta g, U += g (and the bias) in the epilogue        M = o, N = k, K = b
// The accumulator tile of BWD_WEIGHT is applied to W and U directly: g never goes to memory.
#include "aet_device.h"
#include "aet_internal.h"

namespace aet {

typedef float f4 __attribute__((ext_vector_type(4)));

enum { DENSE_FWD = 0, DENSE_BWD_DATA = 1, DENSE_BWD_WEIGHT = 2 };

constexpr int kDT = 64;   // output tile edge
constexpr int kDK = 32;   // contraction chunk

// NTW: N tiles (of 16) per workgroup: 4 (each wave owns one N tile and all four M tiles).
template <int MODE, int NTW>
__global__ void __launch_bounds__(256)
k_dense_mfma(const RoundParams *__restrict__ rp, int u, int B, int K, int O, int64_t w_off,
             int64_t b_off, int relu, const float *__restrict__ x, const float *__restrict__ y,
             float *__restrict__ z, const float *__restrict__ mask_src) {
    // x: in (FWD, BWD_WEIGHT) or dout (BWD_DATA); y: dout (BWD_WEIGHT); z: out / din
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 15, lg = lane >> 4;
    const gcf_ptr W = as_global(p.W) + w_off;
    const int64_t cb = (int64_t)blockIdx.z * B;  // first sample of this client in the scratch

    // GEMM extents
    const int M = MODE == DENSE_BWD_WEIGHT ? O : B;
    const int N = MODE == DENSE_FWD ? O : K;
    const int KD = MODE == DENSE_FWD ? K : (MODE == DENSE_BWD_DATA ? O : B);
    constexpr int NW = 16 * NTW;  // columns per workgroup
    const int m0 = blockIdx.y * kDT, n0 = blockIdx.x * NW;

    __shared__ float As[kDT][kDK + 1];   // As[m][kk]
    __shared__ float Bs[kDK][NW + 1];    // Bs[kk][n]

    // element (m, kd) of the left operand and (kd, n) of the right one, zero outside
    auto left = [&](int m, int kd) -> float {
        if (m >= M || kd >= KD) return 0.f;
        if (MODE == DENSE_FWD) return as_global(x)[(cb + m) * K + kd];          // in[b][k]
        if (MODE == DENSE_BWD_DATA) return as_global(x)[(cb + m) * O + kd];     // dout[b][o]
        return as_global(y)[(cb + kd) * O + m];                                  // dout[b][o], m = o
    };
    auto right = [&](int kd, int n) -> float {
        if (n >= N || kd >= KD) return 0.f;
        if (MODE == DENSE_FWD) return W[(int64_t)n * K + kd];                   // W[o][k]
        if (MODE == DENSE_BWD_DATA) return W[(int64_t)kd * K + n];              // W[o][k], n = k
        return as_global(x)[(cb + kd) * K + n];                                  // in[b][k]
    };

    constexpr int MA = NTW == 4 ? 4 : 1;  // accumulator tiles per wave
    const int ntile = NTW == 4 ? wave : 0;
    f4 acc[MA];
#pragma unroll
    for (int m = 0; m < MA; ++m) acc[m] = f4{0.f, 0.f, 0.f, 0.f};

    for (int k0 = 0; k0 < KD; k0 += kDK) {
        __syncthreads();
        // stage with the thread index running along the dimension that is contiguous in memory
        if (MODE == DENSE_BWD_WEIGHT) {
            for (int e = tid; e < kDT * kDK; e += 256) {  // m fastest
                const int kk = e / kDT, m = e - kk * kDT;
                As[m][kk] = left(m0 + m, k0 + kk);
            }
        } else {
            for (int e = tid; e < kDT * kDK; e += 256) {  // kd fastest
                const int m = e / kDK, kk = e - m * kDK;
                As[m][kk] = left(m0 + m, k0 + kk);
            }
        }
        if (MODE == DENSE_FWD) {
            for (int e = tid; e < NW * kDK; e += 256) {  // kd fastest
                const int n = e / kDK, kk = e - n * kDK;
                Bs[kk][n] = right(k0 + kk, n0 + n);
            }
        } else {
            for (int e = tid; e < NW * kDK; e += 256) {  // n fastest
                const int kk = e / NW, n = e - kk * NW;
                Bs[kk][n] = right(k0 + kk, n0 + n);
            }
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < kDK / 4; ++s) {
            const float b = Bs[4 * s + lg][16 * ntile + li];
#pragma unroll
            for (int m = 0; m < MA; ++m) {
                const int mt = NTW == 4 ? m : wave;
                acc[m] = __builtin_amdgcn_mfma_f32_16x16x4f32(As[16 * mt + li][4 * s + lg], b, acc[m], 0, 0, 0);
            }
        }
    }

    // epilogue: lane holds column n = n0 + 16*wave + li and rows m = m0 + 16*mt + 4*lg + r
    const int n = n0 + 16 * ntile + li;
    if (MODE == DENSE_BWD_WEIGHT) {
        const float invB = 1.0f / (float)B;
        const gf_ptr Wc = as_global(p.W), Uc = as_global(p.U);
        if (n < N) {
#pragma unroll
            for (int m = 0; m < MA; ++m)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int o = m0 + 16 * (NTW == 4 ? m : wave) + 4 * lg + r;
                    if (o < M) {
                        const float g = acc[m][r] * invB;
                        const int64_t wi = w_off + (int64_t)o * K + n;
                        Wc[wi] -= p.eta * g;
                        Uc[wi] += g;
                    }
                }
        }
        // bias: the first column block sums dout over the mini-batch
        if (blockIdx.x == 0 && tid < kDT && m0 + tid < O) {
            const int o = m0 + tid;
            float s = 0.f;
#pragma unroll 8
            for (int b = 0; b < B; ++b) s += as_global(y)[(cb + b) * O + o];
            s *= invB;
            Wc[b_off + o] -= p.eta * s;
            Uc[b_off + o] += s;
        }
    } else {
        const gf_ptr zg = as_global(z);
        if (n < N) {
            const float bias = MODE == DENSE_FWD ? as_global(p.W)[b_off + n] : 0.f;
#pragma unroll
            for (int m = 0; m < MA; ++m)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int b = m0 + 16 * (NTW == 4 ? m : wave) + 4 * lg + r;
                    if (b < M) {
                        float v = acc[m][r] + bias;
                        const int64_t i = (cb + b) * N + n;
                        if (MODE == DENSE_FWD) {
                            if (relu && !(v > 0.f)) v = 0.f;
                        } else if (mask_src && !(as_global(mask_src)[i] > 0.f)) {
                            v = 0.f;
                        }
                        zg[i] = v;
                    }
                }
        }
    }
}

// Backward-weight with vector memory accesses, for layers whose rows are 16-byte aligned
// (K and the parameter offset multiples of 4).  The GEMM is taken transposed,
//   g^T[k][o] = (1/B) sum_b in[b][k] dout[b][o],        M = k, N = o, contraction over b,
// so that the four accumulator elements of a lane are four consecutive k of one output
// unit o: W and U are updated in place with float4 loads and stores.  A workgroup owns 64
// k x 64 o; wave w owns the 16 output units 16w.. and all four k tiles.  Both operands are
// staged as [b][k] / [b][o] rows (float4 loads without branches: what lies outside is read
// from a valid dummy address and replaced by zero), row stride 80 floats = 16 mod 32 banks.
// VO: dout rows are 16-byte aligned too (O a multiple of 4).
constexpr int kWS = 80;   // LDS row stride of the staged operands

template <bool VO>
__global__ void __launch_bounds__(256)
k_dense_wgrad(const RoundParams *__restrict__ rp, int u, int B, int K, int O, int64_t w_off,
              int64_t b_off, const float *__restrict__ x, const float *__restrict__ y) {
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 15, lg = lane >> 4;
    const int kbase = blockIdx.x * kDT, obase = blockIdx.y * kDT;
    const int64_t cb = (int64_t)blockIdx.z * B;
    typedef const f4 __attribute__((address_space(1))) *gv4;
    typedef f4 __attribute__((address_space(1))) *gw4;
    const gcf_ptr xin = as_global(x) + cb * K;    // in[b][k] of this client
    const gcf_ptr yd = as_global(y) + cb * O;     // dout[b][o]

    __shared__ __attribute__((aligned(16))) float As[kDK * kWS];   // As[b][k]
    __shared__ __attribute__((aligned(16))) float Bs[kDK * kWS];   // Bs[b][o]

    const int srow = tid >> 4, sc4 = 4 * (tid & 15);   // staging: rows srow, srow + 16; 4 columns from sc4
    const bool kok = kbase + sc4 < K;
    const bool ook = obase + sc4 < O;
    const int orow = tid >> 6, ocol = tid & 63;        // scalar staging of dout: rows orow + 4 i

    f4 acc[4];
#pragma unroll
    for (int m = 0; m < 4; ++m) acc[m] = f4{0.f, 0.f, 0.f, 0.f};
    float bsum = 0.f;

    // lane: output unit o = obase + 16 wave + li, k = kbase + 16 m + 4 lg .. + 3.  Its weights
    // and gradient sums are fetched now (nobody else touches them) and are there when the
    // products are done: one memory round trip less at the end.
    const gf_ptr Wc = as_global(p.W), Uc = as_global(p.U);
    const int o = obase + 16 * wave + li;
    f4 wv[4], uv[4];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const int k = kbase + 16 * m + 4 * lg;
        const bool ok = o < O && k < K;
        const int64_t wi = ok ? w_off + (int64_t)o * K + k : w_off;
        wv[m] = *reinterpret_cast<gv4>(Wc + wi);
        uv[m] = *reinterpret_cast<gv4>(Uc + wi);
    }

    for (int b0 = 0; b0 < B; b0 += kDK) {
        __syncthreads();
        f4 va[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int b = b0 + srow + 16 * i;
            const bool ok = kok && b < B;
            va[i] = *reinterpret_cast<gv4>(xin + (ok ? (int64_t)b * K + kbase + sc4 : 0));
            if (!ok) va[i] = f4{0.f, 0.f, 0.f, 0.f};
        }
        if (VO) {
            f4 vb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int b = b0 + srow + 16 * i;
                const bool ok = ook && b < B;
                vb[i] = *reinterpret_cast<gv4>(yd + (ok ? (int64_t)b * O + obase + sc4 : 0));
                if (!ok) vb[i] = f4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) *reinterpret_cast<f4 *>(&Bs[(srow + 16 * i) * kWS + sc4]) = vb[i];
        } else {
            float vb[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int b = b0 + orow + 4 * i;
                const bool ok = obase + ocol < O && b < B;
                vb[i] = yd[ok ? (int64_t)b * O + obase + ocol : 0];
                if (!ok) vb[i] = 0.f;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) Bs[(orow + 4 * i) * kWS + ocol] = vb[i];
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) *reinterpret_cast<f4 *>(&As[(srow + 16 * i) * kWS + sc4]) = va[i];
        __syncthreads();
#pragma unroll
        for (int s = 0; s < kDK / 4; ++s) {
            const float b = Bs[(4 * s + lg) * kWS + 16 * wave + li];
#pragma unroll
            for (int m = 0; m < 4; ++m)
                acc[m] = __builtin_amdgcn_mfma_f32_16x16x4f32(As[(4 * s + lg) * kWS + 16 * m + li], b, acc[m], 0, 0, 0);
        }
        // bias gradient: the first k block sums the staged dout over the mini-batch (rows
        // beyond the mini-batch are zero)
        if (blockIdx.x == 0 && tid < kDT) {
#pragma unroll
            for (int b = 0; b < kDK; ++b) bsum += Bs[b * kWS + tid];
        }
    }

    const float invB = 1.0f / (float)B;
    if (o < O) {
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const int k = kbase + 16 * m + 4 * lg;
            if (k < K) {
                const int64_t wi = w_off + (int64_t)o * K + k;
                const f4 g = acc[m] * invB;
                *reinterpret_cast<gw4>(Wc + wi) = wv[m] - p.eta * g;
                *reinterpret_cast<gw4>(Uc + wi) = uv[m] + g;
            }
        }
    }
    if (blockIdx.x == 0 && tid < kDT && obase + tid < O) {
        const int ob = obase + tid;
        const float sb = bsum * invB;
        Wc[b_off + ob] -= p.eta * sb;
        Uc[b_off + ob] += sb;
    }
}

// Backward-data with vector memory accesses, for layers whose rows are 16-byte aligned (K and
// the parameter offset multiples of 4).  The GEMM is taken transposed,
//   din^T[k][b] = sum_o W[o][k] dout[b][o],             M = k, N = b, contraction over o,
// so that W is staged as it lies in memory (rows of consecutive k) and a lane ends up with
// four consecutive k of one sample: float4 stores (and float4 loads of the ReLU mask).
// A workgroup owns 64 k x 16*NBT samples; wave w owns the k tile 16w.. and all sample tiles.
// dout is staged transposed ([o][b], odd row stride); chunks of 32 output units.
template <int NBT>
__global__ void __launch_bounds__(256)
k_dense_dgrad(const RoundParams *__restrict__ rp, int u, int B, int K, int O, int64_t w_off,
              const float *__restrict__ y, float *__restrict__ z, const float *__restrict__ mask_src) {
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    constexpr int BS = NBT == 4 ? 81 : 49;   // row stride of the transposed dout tile
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 15, lg = lane >> 4;
    const int kbase = blockIdx.x * kDT, bbase = blockIdx.y * 16 * NBT;
    const int64_t cb = (int64_t)blockIdx.z * B;
    typedef const f4 __attribute__((address_space(1))) *gv4;
    typedef f4 __attribute__((address_space(1))) *gw4;
    const gcf_ptr W = as_global(p.W) + w_off;
    const gcf_ptr yd = as_global(y) + cb * O;     // dout[b][o] of this client

    __shared__ __attribute__((aligned(16))) float As[kDK * kWS];   // As[o][k]
    __shared__ float Bs[kDK * BS];                                 // Bs[o][b]

    const int srow = tid >> 4, sc4 = 4 * (tid & 15);   // W: rows srow, srow + 16; 4 columns from sc4
    const bool kok = kbase + sc4 < K;
    const int oo = tid & 31, brow = tid >> 5;          // dout: unit oo of the chunk, samples brow + 8 i

    f4 acc[NBT];
#pragma unroll
    for (int n = 0; n < NBT; ++n) acc[n] = f4{0.f, 0.f, 0.f, 0.f};

    for (int o0 = 0; o0 < O; o0 += kDK) {
        __syncthreads();
        f4 va[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int o = o0 + srow + 16 * i;
            const bool ok = kok && o < O;
            va[i] = *reinterpret_cast<gv4>(W + (ok ? (int64_t)o * K + kbase + sc4 : 0));
            if (!ok) va[i] = f4{0.f, 0.f, 0.f, 0.f};
        }
        float vb[2 * NBT];
#pragma unroll
        for (int i = 0; i < 2 * NBT; ++i) {
            const int b = bbase + brow + 8 * i;
            const bool ok = o0 + oo < O && b < B;
            vb[i] = yd[ok ? (int64_t)b * O + o0 + oo : 0];
            if (!ok) vb[i] = 0.f;
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) *reinterpret_cast<f4 *>(&As[(srow + 16 * i) * kWS + sc4]) = va[i];
#pragma unroll
        for (int i = 0; i < 2 * NBT; ++i) Bs[oo * BS + brow + 8 * i] = vb[i];
        __syncthreads();
#pragma unroll
        for (int s = 0; s < kDK / 4; ++s) {
            const float a = As[(4 * s + lg) * kWS + 16 * wave + li];
#pragma unroll
            for (int n = 0; n < NBT; ++n)
                acc[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, Bs[(4 * s + lg) * BS + 16 * n + li], acc[n], 0, 0, 0);
        }
    }

    // lane: k = kbase + 16 wave + 4 lg .. + 3, sample b = bbase + 16 n + li
    const int k = kbase + 16 * wave + 4 * lg;
    if (k < K) {
#pragma unroll
        for (int n = 0; n < NBT; ++n) {
            const int b = bbase + 16 * n + li;
            if (b < B) {
                const int64_t i = (cb + b) * K + k;
                f4 v = acc[n];
                if (mask_src) {
                    const f4 mk = *reinterpret_cast<gv4>(as_global(mask_src) + i);
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (!(mk[r] > 0.f)) v[r] = 0.f;
                }
                *reinterpret_cast<gw4>(as_global(z) + i) = v;
            }
        }
    }
}

// Forward pass of a layer with few output tiles (small mini-batch, moderate width): one
// workgroup per 16 x 16 output tile, its 4 waves split the contraction (wave w takes the
// 16-wide chunks w, w+4, ...) and feed the matrix cores straight from global memory: lane
// (li, lg) loads the four consecutive k = 16c + 4lg .. 4lg+3 of row li of both operands, and
// product r of the chunk contracts the r-th of them (the order of k inside a chunk is free
// as long as both operands agree).  The four partial tiles are added in wave order in LDS.
// MB: 16-sample tiles per workgroup (1 or 4); the tiles share the loads of the weight rows.
template <bool VEC, int MB>
__global__ void __launch_bounds__(256)
k_dense_fwd_direct(const RoundParams *__restrict__ rp, int u, int B, int K, int O, int64_t w_off,
                   int64_t b_off, int relu, const float *__restrict__ x, float *__restrict__ z) {
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 15, lg = lane >> 4;
    const int n0 = blockIdx.x * 16, m0 = blockIdx.y * 16 * MB;
    const int64_t cb = (int64_t)blockIdx.z * B;
    const bool brow = n0 + li < O;
    bool arow[MB];
    gcf_ptr ap[MB];
#pragma unroll
    for (int t = 0; t < MB; ++t) {
        arow[t] = m0 + 16 * t + li < B;
        ap[t] = as_global(x) + (cb + (arow[t] ? m0 + 16 * t + li : 0)) * K + 4 * lg;
    }
    const gcf_ptr bp = as_global(p.W) + w_off + (int64_t)(brow ? n0 + li : 0) * K + 4 * lg;
    typedef const f4 __attribute__((address_space(1))) *gv4;

    auto load = [&](gcf_ptr q, bool row, int k) -> f4 {   // k = first of the lane's four
        f4 v = {0.f, 0.f, 0.f, 0.f};
        if (!row) return v;
        if (VEC) {
            if (k + 3 < K) v = *reinterpret_cast<gv4>(q);
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (k + r < K) v[r] = q[r];
        }
        return v;
    };

    f4 acc[MB];
#pragma unroll
    for (int t = 0; t < MB; ++t) acc[t] = f4{0.f, 0.f, 0.f, 0.f};
    constexpr int UN = 4;   // chunks in flight per wave
    const int nchunk = (K + 15) / 16;
    for (int c0 = wave; c0 < nchunk; c0 += 4 * UN) {
        f4 a[UN][MB], b[UN];
#pragma unroll
        for (int j = 0; j < UN; ++j) {
            const int c = c0 + 4 * j;
            b[j] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < MB; ++t) a[j][t] = b[j];
            if (c < nchunk) {
#pragma unroll
                for (int t = 0; t < MB; ++t) a[j][t] = load(ap[t] + 16 * c, arow[t], 16 * c + 4 * lg);
                b[j] = load(bp + 16 * c, brow, 16 * c + 4 * lg);
            }
        }
#pragma unroll
        for (int j = 0; j < UN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int t = 0; t < MB; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[j][t][r], b[j][r], acc[t], 0, 0, 0);
    }
    __shared__ float part[4][16 * MB][17];
#pragma unroll
    for (int t = 0; t < MB; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) part[wave][16 * t + 4 * lg + r][li] = acc[t][r];   // (sample, feature)
    __syncthreads();
#pragma unroll
    for (int t = 0; t < MB; ++t) {
        const int b = 16 * t + (tid >> 4), o = tid & 15;   // 256 threads = one 16 x 16 tile
        if (m0 + b < B && n0 + o < O) {
            float v = as_global(p.W)[b_off + n0 + o];
            v += part[0][b][o];
            v += part[1][b][o];
            v += part[2][b][o];
            v += part[3][b][o];
            if (relu && !(v > 0.f)) v = 0.f;
            as_global(z)[(cb + m0 + b) * O + n0 + o] = v;
        }
    }
}

hipError_t launch_dense_mfma(hipStream_t s, Profiler *prof, int mode, const RoundParams *dp, int nact,
                             int u, int B, int K, int O, int64_t w_off, int64_t b_off, int relu,
                             const float *x, const float *y, float *z, const float *mask_src) {
    const int M = mode == DENSE_BWD_WEIGHT ? O : B;
    const int N = mode == DENSE_FWD ? O : K;
    // forward pass: 16 x 16 tiles straight from global memory when the wide tiling would leave
    // most of the GPU idle
    const bool narrow = mode == DENSE_FWD && (int64_t)((N + kDT - 1) / kDT) * ((M + kDT - 1) / kDT) * nact < 512;
    const int nw = narrow ? 16 : kDT;
    dim3 grid((unsigned)((N + nw - 1) / nw), (unsigned)((M + kDT - 1) / kDT), (unsigned)nact);
    const int fam = mode == DENSE_FWD ? F_DENSE_FWD : mode == DENSE_BWD_DATA ? F_DENSE_BWD_DATA : F_DENSE_BWD_WEIGHT;
    const bool timed = prof && prof->on[fam];
    if (timed) prof->before(fam, s);
    if (mode == DENSE_FWD && narrow) {
        // float4 loads need 16-byte aligned rows: K a multiple of 4 (all offsets are multiples
        // of 64 floats otherwise) and the parameter offset a multiple of 4
        const bool vec = (K & 3) == 0 && (w_off & 3) == 0;
        // four sample tiles per workgroup share the weight rows, but only when that still
        // gives every compute unit two workgroups; otherwise one tile each
        if (M > 16 && (int64_t)((N + 15) / 16) * ((M + 63) / 64) * nact >= 512) {
            dim3 dgrid((unsigned)((N + 15) / 16), (unsigned)((M + 63) / 64), (unsigned)nact);
            if (vec) k_dense_fwd_direct<true, 4><<<dgrid, 256, 0, s>>>(dp, u, B, K, O, w_off, b_off, relu, x, z);
            else k_dense_fwd_direct<false, 4><<<dgrid, 256, 0, s>>>(dp, u, B, K, O, w_off, b_off, relu, x, z);
        } else {
            dim3 dgrid((unsigned)((N + 15) / 16), (unsigned)((M + 15) / 16), (unsigned)nact);
            if (vec) k_dense_fwd_direct<true, 1><<<dgrid, 256, 0, s>>>(dp, u, B, K, O, w_off, b_off, relu, x, z);
            else k_dense_fwd_direct<false, 1><<<dgrid, 256, 0, s>>>(dp, u, B, K, O, w_off, b_off, relu, x, z);
        }
    } else if (mode == DENSE_FWD)
        k_dense_mfma<DENSE_FWD, 4><<<grid, 256, 0, s>>>(dp, u, B, K, O, w_off, b_off, relu, x, y, z, mask_src);
    else if (mode == DENSE_BWD_DATA && (K & 3) == 0 && (w_off & 3) == 0) {
        const int nbt = B <= 16 ? 1 : B <= 32 ? 2 : 4;
        dim3 dgrid((unsigned)((K + kDT - 1) / kDT), (unsigned)((B + 16 * nbt - 1) / (16 * nbt)), (unsigned)nact);
        if (nbt == 1) k_dense_dgrad<1><<<dgrid, 256, 0, s>>>(dp, u, B, K, O, w_off, x, z, mask_src);
        else if (nbt == 2) k_dense_dgrad<2><<<dgrid, 256, 0, s>>>(dp, u, B, K, O, w_off, x, z, mask_src);
        else k_dense_dgrad<4><<<dgrid, 256, 0, s>>>(dp, u, B, K, O, w_off, x, z, mask_src);
    } else if (mode == DENSE_BWD_DATA)
        k_dense_mfma<DENSE_BWD_DATA, 4><<<grid, 256, 0, s>>>(dp, u, B, K, O, w_off, b_off, relu, x, y, z, mask_src);
    else if ((K & 3) == 0 && (w_off & 3) == 0) {
        dim3 wgrid((unsigned)((K + kDT - 1) / kDT), (unsigned)((O + kDT - 1) / kDT), (unsigned)nact);
        if ((O & 3) == 0) k_dense_wgrad<true><<<wgrid, 256, 0, s>>>(dp, u, B, K, O, w_off, b_off, x, y);
        else k_dense_wgrad<false><<<wgrid, 256, 0, s>>>(dp, u, B, K, O, w_off, b_off, x, y);
    } else
        k_dense_mfma<DENSE_BWD_WEIGHT, 4><<<grid, 256, 0, s>>>(dp, u, B, K, O, w_off, b_off, relu, x, y, z, mask_src);
    if (timed) prof->after(fam, s);
    return hipGetLastError();
}

}  // namespace aet
