// Fused local round for LeNet-5-style models:
//   conv 5x5 (1 -> 6, ReLU), 2x2 max pool, conv 5x5 (6 -> 16, ReLU), 2x2 max pool,
//   dense F0 -> 120 (ReLU), dense 120 -> 84 (ReLU), dense 84 -> 10, mini-batch B = 16.
//
// One launch runs the whole round (Algorithm 2, MainComputeNode: all s_i/B recursions) of
// every active client.  A client is a cluster of 4 workgroups.  Workgroup g
//   - runs the convolutional part for samples 4g..4g+3 of every mini-batch, with a full copy
//     of the two filter banks in LDS;
//   - owns 30 of the 120 units of the first dense layer and 21 of the 84 of the second (their
//     weight rows in LDS, for all 16 samples), and a full copy of the last layer.
// The replica and U never leave the chip during the round: weights live in LDS (they are read
// in several patterns), every thread keeps the U entries of the weights it updates in
// registers.  Per recursion the workgroups of a cluster exchange, through tagged 64-bit
// {step, value} words in memory that every reader polls for the current step (no barrier
// across workgroups, no fence):
//   forward   the pooled output of the second convolution, the outputs of the two hidden
//             dense layers (each workgroup posts its samples / units, everyone reads all);
//   backward  partial sums of d loss / d (input) of the two hidden dense layers over the own
//             units (readers add the four partials in workgroup order), and the partial
//             gradients of the two filter banks over the own samples (likewise), after
//             which every workgroup applies the same update to its copy.
// Every exchange involves all four workgroups in both directions, so one record per
// exchange is enough: nobody can post step u+1 of an exchange before everybody has read
// step u of it.
//
// Max pooling keeps, per window, which of its four inputs won; the backward pass through a
// convolution + ReLU + pool stage touches only that input (the other three get no gradient).
// The conv-1 filter gradient is therefore a sum over one position per window (vector ALU); for
// conv 2 the window winners are scattered into a delta map that is zero elsewhere, and the
// filter gradient and the backward-data pass are dense products over it.
//
// The second convolution (forward, filter gradient, backward-data) and the products of the two
// hidden dense layers (forward, backward-data, weight gradient) run on the matrix cores
// (fp32 16 x 16 x 4 products); the first convolution (6 channels) and the 10-class layer on
// the vector ALU.
//
// All workgroups of a client must be resident together; the wait for a peer's word is
// bounded and raises an error flag instead of hanging (every workgroup still runs to the end).
#include <type_traits>

#include "aet_device.h"
#include "aet_internal.h"

namespace aet {

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned long long u64;

constexpr int kLnThreads = 512;
constexpr int kLnG = 4;              // workgroups per client
constexpr int kLnB = 16;             // mini-batch
constexpr int kF1 = 120, kF2 = 84, kNC = 10;
constexpr int kU1 = kF1 / kLnG, kU2 = kF2 / kLnG;   // units of the hidden layers per workgroup
constexpr int kS1 = 124, kS2 = 88;   // LDS row strides of arrays with 120 / 84 columns
constexpr int kWS = 164;              // LDS row stride of the conv-2 filters (150 used; 4 mod 32: the rows of 8 channels cover all banks)
constexpr int kDP = 32 * 17;         // floats of one wave's slice of partial dense outputs
constexpr int kConvP = 2572;         // parameters of the two filter banks (150 + 6 + 2400 + 16)
constexpr int kLnSpin = 1 << 22;     // bounded wait of the exchange poll

// exchange records of one client, in 64-bit words
constexpr int kXA1 = 0;              // [16][256]      pooled output of conv 2
constexpr int kXA2 = 4096;           // [16][128]      output of dense 1
constexpr int kXA3 = 6144;           // [16][96]       output of dense 2
constexpr int kXB1 = 7680;           // [4][16][128]   partial d loss / d (output of dense 1)
constexpr int kXB2 = 15872;          // [4][16][256]   partial d loss / d (pooled output of conv 2)
constexpr int kXB3 = 32256;          // [4][2576]      partial filter-bank gradients
constexpr int kXWords = 43008;

struct LenetDims {
    int H0, P1, H2, P2, F0, lgF0;    // input side, sides after pool 1 / conv 2 / pool 2, F0 = 16 P2^2 = 2^lgF0
    int64_t o_f1, o_f2, o_f3;        // offsets of the dense layers in the flat parameter vector
};

__device__ __forceinline__ float row16_sum_ln(float v) {
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));
    return v;
}
__device__ __forceinline__ float row16_max_ln(float v) {
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true)));
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true)));
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true)));
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true)));
    return v;
}

// Hides a value from the optimiser so that what is derived from it is computed where it is used.
__device__ __forceinline__ int opaque(int x) {
    asm volatile("" : "+v"(x));
    return x;
}

__device__ __forceinline__ void xpost(u64 *p, uint32_t tag, float v) {
    __hip_atomic_store(p, ((u64)tag << 32) | (u64)__float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

struct Waiter {
    uint32_t tag;
    int *errflag;
    bool dead;
};

// N words at once (the loads are in flight together); repeated until every needed word shows
// the current step.  Words that are not needed still point at valid memory.
template <int N>
__device__ __forceinline__ void xfetch(const u64 *(&p)[N], const bool (&need)[N], float (&out)[N], Waiter &w) {
    int spins = 0;
    for (;;) {
        u64 v[N];
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = __hip_atomic_load(p[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        bool ok = true;
#pragma unroll
        for (int i = 0; i < N; ++i) ok = ok && (!need[i] || (uint32_t)(v[i] >> 32) == w.tag);
        if (ok || w.dead) {
#pragma unroll
            for (int i = 0; i < N; ++i) out[i] = __uint_as_float((uint32_t)v[i]);
            return;
        }
        __builtin_amdgcn_s_sleep(1);
        if ((++spins & 255) == 0) {
            if (spins >= kLnSpin || __hip_atomic_load(w.errflag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                __hip_atomic_store(w.errflag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                w.dead = true;
            }
        }
    }
}

// 5 x 5 convolution at the four positions of a 2 x 2 window from a 6 x 6 patch, added to acc
// (the 25 weights are fetched together: fetched one by one next to their products, every
// fetch would wait out its own LDS round trip)
__device__ __forceinline__ void conv_window(const float (&patch)[6][6], const float *__restrict__ wv, float (&acc)[4]) {
    float w[25];
#pragma unroll
    for (int i = 0; i < 25; ++i) w[i] = wv[i];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ky = 0; ky < 5; ++ky)
#pragma unroll
        for (int kx = 0; kx < 5; ++kx) {
            const float wgt = w[ky * 5 + kx];
            acc[0] += wgt * patch[ky][kx];
            acc[1] += wgt * patch[ky][kx + 1];
            acc[2] += wgt * patch[ky + 1][kx];
            acc[3] += wgt * patch[ky + 1][kx + 1];
        }
}
// ReLU, then the first maximum of the window in row-major order
__device__ __forceinline__ float relu_pool(const float (&acc)[4], int &which) {
    float best = acc[0] > 0.f ? acc[0] : 0.f;
    which = 0;
#pragma unroll
    for (int k = 1; k < 4; ++k) {
        const float v = acc[k] > 0.f ? acc[k] : 0.f;
        if (v > best) { best = v; which = k; }
    }
    return best;
}

// G28: the geometry of the 28 x 28 input (12 x 12 pooled maps, 8 x 8 conv-2 maps, 256 features)
// as compile-time constants, so that the operand addresses of the convolution phases are
// immediates; other input sizes take the sizes from d.
template <bool G28>
__global__ void __launch_bounds__(kLnThreads, 1)
k_lenet_round(const RoundParams *__restrict__ rp, int nhere, int rec0, const float *Wg, const LenetDims d,
              u64 *__restrict__ xrec, uint32_t tag0, int *__restrict__ errflag) {
    // consecutive workgroup ids go round the 8 XCDs: the four workgroups of a client get ids
    // that land on the same XCD and exchange through its L2
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int a = xcd + 8 * (slot / kLnG), g = slot % kLnG;
    if (a >= nhere) return;
    const RoundParams p = rp[a];
    const gcf_ptr Xg = as_global(p.X);
    const gci_ptr yg = as_global(p.y);
    const gf_ptr Wc = as_global(p.W), Uc = as_global(p.U);
    const int tid = threadIdx.x;
    const int H0 = G28 ? 28 : d.H0, P1 = G28 ? 12 : d.P1, H2 = G28 ? 8 : d.H2, P2 = G28 ? 4 : d.P2, F0 = G28 ? 256 : d.F0;
    const int lgF0 = G28 ? 8 : d.lgF0;
    const int nwin1 = P1 * P1, nwin2 = P2 * P2, npix = H0 * H0;
    const int P1S = 6 * nwin1 + 8;       // per-sample stride of the pooled conv-1 maps
    const int F0P = F0 + 4;              // row stride of arrays with F0 columns
    const float invB = 1.0f / (float)kLnB;
    const float eta = p.eta;

    extern __shared__ __align__(16) float smem[];
    auto up4 = [](int n) { return (n + 3) & ~3; };
    float *xs = smem;                              // [4][npix]          own samples
    float *p1 = xs + up4(4 * npix);                // [4][P1S]           pooled conv 1 (after ReLU)
    float *a0 = p1 + 4 * P1S;                      // [16][F0P]          pooled conv 2, all samples
    float *d2own = a0 + 16 * F0P;                  // [16][24]   delta of the own units of dense 2
    float *d1own = d2own + 16 * 24;                // [32][16]   ... of dense 1, unit-major
    // the winner of every pooling window, as the offset of that input inside its map
    uint16_t *off1 = reinterpret_cast<uint16_t *>(d1own + 16 * 32);        // [4][6][nwin1] in the H0 x H0 image (top-left of the 5 x 5 patch)
    uint16_t *off2 = off1 + up4(4 * 6 * nwin1);                          // [4][F0]       in the P1 x P1 pooled conv-1 map
    uint8_t *pos2 = reinterpret_cast<uint8_t *>(off2 + up4(4 * F0));     // [4][F0]       in the H2 x H2 conv-2 map
    float *wc1 = reinterpret_cast<float *>(pos2 + up4(4 * F0));          // [150] + bias [6] (+ pad)
    float *wc2 = wc1 + 160;                        // [16][kWS]
    float *wc2b = wc2 + 16 * kWS;                  // [16]
    float *w1s = wc2b + 16;                        // [30][F0P]
    float *b1s = w1s + kU1 * F0P;                  // [32]
    float *w2s = b1s + 32;                         // [21][kS1]
    float *b2s = w2s + kU2 * kS1;                  // [32]
    float *w3s = b2s + 32;                         // [10][kS2]
    float *b3s = w3s + kNC * kS2;                  // [16]
    float *h1 = b3s + 16;                          // [16][kS1]
    float *h2 = h1 + 16 * kS1;                     // [16][kS2]
    float *dz = h2 + 16 * kS2;                     // [16][16]   d loss / d logits
    float *dp2 = dz + 256 + 16 * kS2;              // (16 x kS2 floats of room in front: dp1 reaches into them)                   // [4][F0]    delta at the pooled conv-2 outputs (own samples)
    float *gsum = dp2 + up4(4 * F0);               // [2576]     filter-bank gradients over the own samples
    float *c1part = gsum + 2576;                   // [14][160]  conv-1 gradient, partial over window groups
    float *lossb = c1part + 14 * 160;              // [16]
    int *labs = reinterpret_cast<int *>(lossb + 16);   // [16]
    float *lossacc = reinterpret_cast<float *>(labs + 16);  // [4]
    // regions that are dead by the time these are needed
    float *dc2 = a0;                               // [4][16][CS2]    delta at the conv-2 outputs, over a0 .. d1own (after the dense backward)
    const int CS2 = H2 * H2 + 4;                   // its channel stride: the rows of consecutive channels start 4 banks apart
    float *dp1 = h1;                               // [4][P1S]        delta at the pooled conv-1 outputs
    float *dpart = gsum;                           // [8][kDP]        partial sums of the dense forward products, one [32 units][17] slice per wave (over gsum, c1part)

    u64 *rec = xrec + (int64_t)(rec0 + a) * kXWords;
    Waiter wt{tag0, errflag, false};

    // ---- adopt the global model (server form) or go on from the own replica (Wg == NULL) ----
    const float *src = Wg ? Wg : p.W;
    for (int i = tid; i < 156; i += kLnThreads) wc1[i] = src[i];
    for (int i = tid; i < 2400; i += kLnThreads) wc2[(i / 150) * kWS + i % 150] = src[156 + i];
    if (tid < 16) wc2b[tid] = src[2556 + tid];
    for (int i = tid; i < kU1 * F0; i += kLnThreads) {
        const int ul = i / F0, k = i % F0;
        w1s[ul * F0P + k] = src[d.o_f1 + (int64_t)(kU1 * g + ul) * F0 + k];
    }
    if (tid < kU1) b1s[tid] = src[d.o_f1 + (int64_t)kF1 * F0 + kU1 * g + tid];
    for (int i = tid; i < kU2 * kF1; i += kLnThreads) {
        const int ul = i / kF1, k = i % kF1;
        w2s[ul * kS1 + k] = src[d.o_f2 + (int64_t)(kU2 * g + ul) * kF1 + k];
    }
    if (tid < kU2) b2s[tid] = src[d.o_f2 + kF2 * kF1 + kU2 * g + tid];
    for (int i = tid; i < kNC * kF2; i += kLnThreads) w3s[(i / kF2) * kS2 + i % kF2] = src[d.o_f3 + i];
    if (tid < kNC) b3s[tid] = src[d.o_f3 + kNC * kF2 + tid];
    if (tid == 0) lossacc[0] = 0.f;
    // U of the weights this thread updates
    float U1[16], U2[8], U3[2], UC[6];
    float U1b = 0.f, U2b = 0.f, U3b = 0.f;
#pragma unroll
    for (int j = 0; j < 16; ++j) U1[j] = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) U2[j] = 0.f;
#pragma unroll
    for (int j = 0; j < 2; ++j) U3[j] = 0.f;
#pragma unroll
    for (int j = 0; j < 6; ++j) UC[j] = 0.f;

    // the own samples' rows travel global -> registers (one recursion ahead) -> LDS
    const int nq = npix >> 2;   // 16-byte pieces per row
    auto load_rows = [&](int u, f4 (&xr)[2], int &lab) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int e = tid + kLnThreads * j;
            xr[j] = f4{0.f, 0.f, 0.f, 0.f};
            if (e < 4 * nq) {
                const int s = e / nq, q = e % nq;
                const uint32_t row = sample_row(p.key, (uint64_t)(p.q0 + (int64_t)u * kLnB + 4 * g + s), p.n_samples);
                xr[j] = *reinterpret_cast<const f4 __attribute__((address_space(1))) *>(Xg + (int64_t)row * npix + 4 * q);
            }
        }
        lab = 0;
        if (tid < kLnB) lab = yg[sample_row(p.key, (uint64_t)(p.q0 + (int64_t)u * kLnB + tid), p.n_samples)];
    };
    auto store_rows = [&](const f4 (&xr)[2], int lab) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int e = tid + kLnThreads * j;
            if (e < 4 * nq) *reinterpret_cast<f4 *>(xs + 4 * e) = xr[j];   // s * npix + 4 q = 4 e
        }
        if (tid < kLnB) labs[tid] = lab;
    };
    f4 xr[2];
    int labr = 0;
    if (p.m > 0) {
        load_rows(0, xr, labr);
        store_rows(xr, labr);
    }
    __syncthreads();

    for (int u = 0; u < p.m; ++u) {
        // index arithmetic is redone where it is used instead of being kept in registers across
        // the whole recursion
        int tq = opaque(tid);
        wt.tag = tag0 + (uint32_t)u;
        const bool more = u + 1 < p.m;
        if (more) load_rows(u + 1, xr, labr);   // Algorithm 2, sampling step: a counter hash, known ahead

        tq = opaque(tq);
        // ---- conv 1 + ReLU + pool: item = (sample, window, three of the six channels) --------
#pragma unroll 1
        for (int it = tq; it < 8 * nwin1; it += kLnThreads) {
            const int half = it & 1, w = it >> 1, px = w % P1, py = (w / P1) % P1, s = w / nwin1;
            float patch[6][6];
            // (H0 is even and the patch starts at an even column: its rows are three aligned pairs)
            typedef float f2 __attribute__((ext_vector_type(2)));
            const float *xp = xs + s * npix + (2 * py) * H0 + 2 * px;
#pragma unroll
            for (int i = 0; i < 6; ++i)
#pragma unroll
                for (int j = 0; j < 6; j += 2) {
                    const f2 v = *reinterpret_cast<const f2 *>(xp + i * H0 + j);
                    patch[i][j] = v[0];
                    patch[i][j + 1] = v[1];
                }
#pragma unroll
            for (int cc = 0; cc < 3; ++cc) {
                const int c = 3 * half + cc;
                const float b = wc1[150 + c];
                float acc[4] = {b, b, b, b};
                conv_window(patch, wc1 + c * 25, acc);
                int which;
                const float v = relu_pool(acc, which);
                p1[s * P1S + c * nwin1 + py * P1 + px] = v;
                off1[(s * 6 + c) * nwin1 + py * P1 + px] = (uint16_t)((2 * py + (which >> 1)) * H0 + 2 * px + (which & 1));
            }
        }
        __syncthreads();

        tq = opaque(tq);
        // ---- conv 2 + ReLU + pool on the matrix cores ------------------------------------------
        // out[c][pos] = sum_k w[c][k] patch[k][pos] as 16 x 16 x 4 products: the rows are the 16
        // channels, the columns 16 output positions (four pooling windows, the four positions
        // of a window in neighbouring lanes), the contraction runs over the 150 (ci, ky, kx)
        // in an order that keeps every operand address "lane constant + step constant":
        //   30 steps (ci, ky) with kx = 0..3 over the four lane groups,
        //    6 steps (ci)     with kx = 4 and ky = 0..3 over the lane groups,
        //    2 steps          with ky = kx = 4 and ci = 0..3 / 4, 5 (two idle groups) over them.
        // A wave takes two tiles at a time (two independent accumulators, one read of the
        // weights).
        {
            const int wave = __builtin_amdgcn_readfirstlane(tq >> 6), lane = tq & 63;
            const int n = lane & 15, kq = lane >> 4;
            const int npos = H2 * H2, ntile = npos >> 2;      // tiles of 16 positions over the 4 own samples
            const float *wa1 = wc2 + n * kWS + kq;
            const float *wa2 = wc2 + n * kWS + 5 * kq + 4;
            const float *wa3 = wc2 + n * kWS + 25 * kq + 24;
            const float *wa4 = wc2 + n * kWS + 25 * (4 + (kq & 1)) + 24;
            const bool last2 = kq < 2;
#pragma unroll 1
            for (int t0 = wave; t0 < ntile; t0 += 2 * (kLnThreads / 64)) {
                const int t1 = t0 + kLnThreads / 64;
                const bool two = t1 < ntile;
                const float *pb[2];
                int sj[2], winj[2], qj[2];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int j = ((h == 0 || two) ? (h == 0 ? t0 : t1) : t0) * 16 + n;
                    const int sl = j / npos, jj = j - sl * npos, win = jj >> 2, q = jj & 3;
                    const int oy = win / P2, ox = win - oy * P2;
                    sj[h] = sl; winj[h] = win; qj[h] = q;
                    pb[h] = p1 + sl * P1S + (2 * oy + (q >> 1)) * P1 + 2 * ox + (q & 1);
                }
                f4 acc[2] = {f4{0.f, 0.f, 0.f, 0.f}, f4{0.f, 0.f, 0.f, 0.f}};
                // operands of the six steps of one input channel (five filter rows with kx < 4,
                // then kx = 4); the next channel's are fetched before the products of the
                // current one are issued
                auto fetch = [&](int ci, float (&wv)[6], float (&bv)[2][6]) {
#pragma unroll
                    for (int ky = 0; ky < 5; ++ky) wv[ky] = wa1[ci * 25 + ky * 5];
                    wv[5] = wa2[ci * 25];
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const float *q1 = pb[h] + ci * nwin1 + kq;
#pragma unroll
                        for (int ky = 0; ky < 5; ++ky) bv[h][ky] = q1[ky * P1];
                        bv[h][5] = pb[h][ci * nwin1 + kq * P1 + 4];
                    }
                };
                auto products = [&](const float (&wv)[6], const float (&bv)[2][6]) {
#pragma unroll
                    for (int ky = 0; ky < 6; ++ky)
#pragma unroll
                        for (int h = 0; h < 2; ++h)
                            acc[h] = __builtin_amdgcn_mfma_f32_16x16x4f32(wv[ky], bv[h][ky], acc[h], 0, 0, 0);
                };
                float wva[6], bva[2][6], wvb[6], bvb[2][6];
                fetch(0, wva, bva);
#pragma unroll 1
                for (int ci = 0; ci < 6; ci += 2) {
                    fetch(ci + 1, wvb, bvb);
                    __builtin_amdgcn_sched_barrier(0);
                    products(wva, bva);
                    __builtin_amdgcn_sched_barrier(0);
                    if (ci + 2 < 6) fetch(ci + 2, wva, bva);
                    __builtin_amdgcn_sched_barrier(0);
                    products(wvb, bvb);
                    __builtin_amdgcn_sched_barrier(0);
                }
                {
                    const float w3 = wa3[0], w4r = wa4[0], w4 = last2 ? w4r : 0.f;
                    float b3[2], b4[2];
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        b3[h] = pb[h][kq * nwin1 + 4 * P1 + 4];
                        b4[h] = pb[h][(4 + (kq & 1)) * nwin1 + 4 * P1 + 4];
                    }
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        acc[h] = __builtin_amdgcn_mfma_f32_16x16x4f32(w3, b3[h], acc[h], 0, 0, 0);
                        acc[h] = __builtin_amdgcn_mfma_f32_16x16x4f32(w4, b4[h], acc[h], 0, 0, 0);
                    }
                }
                // A lane holds position n of the tile for channels 4 kq .. 4 kq + 3.  The four lanes
                // of a window transpose their 4 x 4 values (two exchange steps), after which lane q
                // of the window holds the four positions of channel 4 kq + q: bias, ReLU, the first
                // maximum in row-major order, and the four stores of that output.
                const float bias = wc2b[4 * kq + (n & 3)];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    if (h == 1 && !two) break;
                    const int sl = sj[h], win = winj[h], q = qj[h];
                    const int oy = win / P2, ox = win - oy * P2;
                    float t[4] = {acc[h][0], acc[h][1], acc[h][2], acc[h][3]};
                    {   // exchange with lane q ^ 1 inside the register pairs (0, 1) and (2, 3)
                        const bool odd = q & 1;
#pragma unroll
                        for (int a2 = 0; a2 < 4; a2 += 2) {
                            const float send = odd ? t[a2] : t[a2 + 1];
                            const float got = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0xB1, 0xF, 0xF, true));
                            if (odd) t[a2] = got; else t[a2 + 1] = got;
                        }
                    }
                    {   // exchange with lane q ^ 2 inside the register pairs (0, 2) and (1, 3)
                        const bool up = q & 2;
#pragma unroll
                        for (int a2 = 0; a2 < 2; ++a2) {
                            const float send = up ? t[a2] : t[a2 + 2];
                            const float got = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0x4E, 0xF, 0xF, true));
                            if (up) t[a2] = got; else t[a2 + 2] = got;
                        }
                    }
                    float best = t[0] + bias;
                    best = best > 0.f ? best : 0.f;
                    int which = 0;
#pragma unroll
                    for (int k = 1; k < 4; ++k) {
                        float v = t[k] + bias;
                        v = v > 0.f ? v : 0.f;
                        if (v > best) { best = v; which = k; }
                    }
                    const int c = 4 * kq + q;
                    const int f = c * nwin2 + win;    // flattened C, H, W
                    const int wy = 2 * oy + (which >> 1), wx = 2 * ox + (which & 1);
                    a0[(4 * g + sl) * F0P + f] = best;
                    off2[sl * F0 + f] = (uint16_t)(wy * P1 + wx);
                    pos2[sl * F0 + f] = (uint8_t)(wy * H2 + wx);
                    xpost(rec + kXA1 + (4 * g + sl) * 256 + f, wt.tag, best);
                }
            }
        }
        // the other workgroups' samples
        for (int e0 = tq; e0 < 16 * F0; e0 += 8 * kLnThreads) {
            const u64 *ptr[8];
            bool need[8];
            float val[8];
            int dst[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int e = e0 + kLnThreads * i;
                const bool in = e < 16 * F0;
                const int b = in ? e >> lgF0 : 0, f = in ? e & (F0 - 1) : 0;
                need[i] = in && (b >> 2) != g;
                ptr[i] = rec + kXA1 + b * 256 + f;
                dst[i] = b * F0P + f;
            }
            xfetch<8>(ptr, need, val, wt);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (need[i]) a0[dst[i]] = val[i];
        }
        __syncthreads();

        tq = opaque(tq);
        // ---- dense 1, own units, on the matrix cores: rows = the 16 samples, columns = the 30 own
        // units in two tiles (two idle columns), the F0 inputs dealt over the waves in runs of
        // F0 / 32 steps of four; the waves' partial sums meet in LDS and are added in wave order ------
        {
            const int wave = __builtin_amdgcn_readfirstlane(tq >> 6), lane = tq & 63;
            const int n = lane & 15, kq = lane >> 4;
            const int nstep = F0 >> 2, per = (nstep + 7) >> 3;      // steps in all, steps per wave
            const int t0 = wave * per, t1 = t0 + per < nstep ? t0 + per : nstep;
            const float *ap = a0 + n * F0P + kq;
            const float *bp0 = w1s + n * F0P + kq, *bp1 = w1s + (16 + n < kU1 ? 16 + n : kU1 - 1) * F0P + kq;
            f4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
            if (F0 == 256) {
                float av[8], b0[8], b1[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    av[i] = ap[4 * (t0 + i)];
                    b0[i] = bp0[4 * (t0 + i)];
                    b1[i] = bp1[4 * (t0 + i)];
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i], b0[i], acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i], b1[i], acc1, 0, 0, 0);
                }
            } else {
#pragma unroll 1
                for (int t = t0; t < t1; ++t) {
                    const float av = ap[4 * t];
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bp0[4 * t], acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bp1[4 * t], acc1, 0, 0, 0);
                }
            }
            // lane: unit n (and 16 + n), samples 4 kq .. 4 kq + 3; unit-major with a stride of 17
            float *dst = dpart + wave * kDP + n * 17 + 4 * kq;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                dst[r] = acc0[r];
                dst[16 * 17 + r] = acc1[r];
            }
        }
        __syncthreads();
        if (tq < kU1 * 16) {
            const int ul = tq >> 4, b = tq & 15;
            float acc = b1s[ul];
#pragma unroll
            for (int w = 0; w < kLnThreads / 64; ++w) acc += dpart[w * kDP + ul * 17 + b];
            const float h = acc > 0.f ? acc : 0.f;
            h1[b * kS1 + kU1 * g + ul] = h;
            xpost(rec + kXA2 + b * 128 + kU1 * g + ul, wt.tag, h);
        }
        for (int e0 = tq; e0 < 16 * kF1; e0 += 4 * kLnThreads) {
            const u64 *ptr[4];
            bool need[4];
            float val[4];
            int dst[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = e0 + kLnThreads * i;
                const bool in = e < 16 * kF1;
                const int b = in ? e / kF1 : 0, k = in ? e % kF1 : 0;
                need[i] = in && k / kU1 != g;
                ptr[i] = rec + kXA2 + b * 128 + k;
                dst[i] = b * kS1 + k;
            }
            xfetch<4>(ptr, need, val, wt);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (need[i]) h1[dst[i]] = val[i];
        }
        __syncthreads();

        tq = opaque(tq);
        // ---- dense 2, own units, on the matrix cores like dense 1: the 30 steps of four inputs are
        // dealt over the waves (four each), the 21 own units fill two column tiles ------------------
        {
            const int wave = __builtin_amdgcn_readfirstlane(tq >> 6), lane = tq & 63;
            const int n = lane & 15, kq = lane >> 4;
            const int t0 = 4 * wave;
            const float *ap = h1 + n * kS1 + kq;
            const float *bp0 = w2s + n * kS1 + kq, *bp1 = w2s + (16 + n < kU2 ? 16 + n : kU2 - 1) * kS1 + kq;
            float av[4], b0[4], b1[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int t = t0 + i < kF1 / 4 ? t0 + i : kF1 / 4 - 1;
                av[i] = ap[4 * t];
                b0[i] = bp0[4 * t];
                b1[i] = bp1[4 * t];
            }
            __builtin_amdgcn_sched_barrier(0);
            f4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (t0 + i < kF1 / 4) {
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i], b0[i], acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i], b1[i], acc1, 0, 0, 0);
                }
            }
            float *dst = dpart + wave * kDP + n * 17 + 4 * kq;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                dst[r] = acc0[r];
                dst[16 * 17 + r] = acc1[r];
            }
        }
        __syncthreads();
        if (tq < kU2 * 16) {
            const int ul = tq >> 4, b = tq & 15;
            float acc = b2s[ul];
#pragma unroll
            for (int w = 0; w < kLnThreads / 64; ++w) acc += dpart[w * kDP + ul * 17 + b];
            const float h = acc > 0.f ? acc : 0.f;
            h2[b * kS2 + kU2 * g + ul] = h;
            xpost(rec + kXA3 + b * 96 + kU2 * g + ul, wt.tag, h);
        }
        for (int e0 = tq; e0 < 16 * kF2; e0 += 4 * kLnThreads) {
            const u64 *ptr[4];
            bool need[4];
            float val[4];
            int dst[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = e0 + kLnThreads * i;
                const bool in = e < 16 * kF2;
                const int b = in ? e / kF2 : 0, k = in ? e % kF2 : 0;
                need[i] = in && k / kU2 != g;
                ptr[i] = rec + kXA3 + b * 96 + k;
                dst[i] = b * kS2 + k;
            }
            xfetch<4>(ptr, need, val, wt);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (need[i]) h2[dst[i]] = val[i];
        }
        __syncthreads();

        tq = opaque(tq);
        // ---- dense 3 (every workgroup, all samples), softmax, d logits: thread = (sample, class) --
        if (tq < 256) {
            const int b = tq >> 4, o = tq & 15;
            float z = 0.f;
            if (o < kNC) {
                f4 part = {b3s[o], 0.f, 0.f, 0.f};
                const float *wr = w3s + o * kS2, *ar = h2 + b * kS2;
#pragma unroll 7
                for (int k = 0; k < kF2; k += 4) {
                    const f4 wv = *reinterpret_cast<const f4 *>(wr + k), av = *reinterpret_cast<const f4 *>(ar + k);
                    part += wv * av;
                }
                z = (part[0] + part[1]) + (part[2] + part[3]);
            }
            const float zmax = row16_max_ln(o < kNC ? z : -3.0e38f);
            const float ex = o < kNC ? __expf(z - zmax) : 0.f;
            const float lse = zmax + __logf(row16_sum_ln(ex));
            const int lab = labs[b];
            if (o == lab) lossb[b] = lse - z;
            dz[b * 16 + o] = o < kNC ? __expf(z - lse) - (o == lab ? 1.f : 0.f) : 0.f;
        }
        __syncthreads();

        tq = opaque(tq);
        // ---- backward through dense 3: only the own units of dense 2 need their delta (reads the
        // not yet updated weights of dense 3) -----------------------------------------------------
        if (tq < kU2 * 16) {
            const int ul = tq >> 4, b = tq & 15, k = kU2 * g + ul;
            float acc = 0.f;
#pragma unroll
            for (int o = 0; o < kNC; ++o) acc += dz[b * 16 + o] * w3s[o * kS2 + k];
            d2own[b * 24 + ul] = h2[b * kS2 + k] > 0.f ? acc : 0.f;
        } else if (tq < kU2 * 16 + 48) {   // columns 21 .. 23: idle steps of the matrix-core product below
            const int i = tq - kU2 * 16;
            d2own[(i & 15) * 24 + kU2 + (i >> 4)] = 0.f;
        }
        if (g == 0 && tq == 511) {
            float s = 0.f;
            for (int b = 0; b < kLnB; ++b) s += lossb[b];
            lossacc[0] += s * invB;
        }
        __syncthreads();

        tq = opaque(tq);
        // ---- backward through dense 2: partial d h1 over the own units -> exchange ---------------
        // on the matrix cores: rows = the 16 samples, columns = the 120 inputs (wave w takes tile
        // w), contraction over the 21 own units in six steps (idle units: zero deltas)
        {
            const int wave = __builtin_amdgcn_readfirstlane(tq >> 6), lane = tq & 63;
            const int n = lane & 15, kq = lane >> 4, k = 16 * wave + n;
            float av[6], bv[6];
#pragma unroll
            for (int t = 0; t < 6; ++t) {
                const int ul = 4 * t + kq, ulc = ul < kU2 ? ul : kU2 - 1;
                av[t] = d2own[n * 24 + ul];
                bv[t] = w2s[ulc * kS1 + k];
            }
            __builtin_amdgcn_sched_barrier(0);
            f4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < 6; ++t) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[t], bv[t], acc, 0, 0, 0);
            if (k < kF1) {
#pragma unroll
                for (int r = 0; r < 4; ++r) xpost(rec + kXB1 + g * 2048 + (4 * kq + r) * 128 + k, wt.tag, acc[r]);
            }
        }
        // dense 3: w <- w - eta g, U <- U + g (the same in every workgroup)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int e = tq + kLnThreads * j;
            if (e < kNC * kF2) {
                const int o = e / kF2, k = e % kF2;
                float s = 0.f;
#pragma unroll
                for (int b = 0; b < kLnB; ++b) s += dz[b * 16 + o] * h2[b * kS2 + k];
                const float gv = s * invB;
                w3s[o * kS2 + k] -= eta * gv;
                U3[j] += gv;
            }
        }
        if (tq < kNC) {
            float s = 0.f;
#pragma unroll
            for (int b = 0; b < kLnB; ++b) s += dz[b * 16 + tq];
            const float gv = s * invB;
            b3s[tq] -= eta * gv;
            U3b += gv;
        }
        __syncthreads();
        // dense 2: g^T = delta^T h1 on the matrix cores (rows = the own units in two tiles, columns =
        // the 120 inputs, wave w takes tile w, contraction over the 16 samples); a lane keeps U of
        // the weights (unit 16 mt + 4 kq + r, input 16 w + n)
        {
            const int wave = __builtin_amdgcn_readfirstlane(tq >> 6), lane = tq & 63;
            const int n = lane & 15, kq = lane >> 4, k = 16 * wave + n;
            float av[2][4], bv[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                av[0][t] = d2own[(4 * t + kq) * 24 + n];
                av[1][t] = d2own[(4 * t + kq) * 24 + (16 + n < 24 ? 16 + n : 23)];
                bv[t] = h1[(4 * t + kq) * kS1 + k];
            }
            __builtin_amdgcn_sched_barrier(0);
            f4 acc[2] = {f4{0.f, 0.f, 0.f, 0.f}, f4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) acc[mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[mt][t], bv[t], acc[mt], 0, 0, 0);
            if (k < kF1) {
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int ul = 16 * mt + 4 * kq + r;
                        if (ul < kU2) {
                            const float gv = acc[mt][r] * invB;
                            w2s[ul * kS1 + k] -= eta * gv;
                            U2[4 * mt + r] += gv;
                        }
                    }
            }
        }
        if (tq < kU2) {
            float s = 0.f;
#pragma unroll
            for (int b = 0; b < kLnB; ++b) s += d2own[b * 24 + tq];
            const float gv = s * invB;
            b2s[tq] -= eta * gv;
            U2b += gv;
        }
        // delta of the own units of dense 1: the four partials in workgroup order
        {
            const bool act = tq < kU1 * 16;
            const int ul = act ? tq >> 4 : 0, b = tq & 15, k = kU1 * g + ul;
            const u64 *ptr[4];
            bool need[4];
            float val[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ptr[i] = rec + kXB1 + i * 2048 + b * 128 + k;
                need[i] = act;
            }
            xfetch<4>(ptr, need, val, wt);
            if (act) {
                float s = val[0];
                s += val[1];
                s += val[2];
                s += val[3];
                d1own[ul * 16 + b] = h1[b * kS1 + k] > 0.f ? s : 0.f;
            } else {
                d1own[tq] = 0.f;   // rows 30 and 31: idle rows of the matrix-core products below
            }
        }
        __syncthreads();

        tq = opaque(tq);
        // ---- backward through dense 1: partial d a0 over the own units -> exchange.  On the matrix
        // cores: rows = the 16 samples, columns = the F0 features in tiles of 16 (tiles w and w + 8
        // for wave w), contraction over the 30 own units in eight steps (the two idle units have
        // zero deltas and read the last weight row) -------------------------------------------------
        {
            const int wave = __builtin_amdgcn_readfirstlane(tq >> 6), lane = tq & 63;
            const int n = lane & 15, kq = lane >> 4;
            const int ntile = F0 >> 4;
            if (wave < ntile) {
                const bool two = wave + 8 < ntile;
                float av[8], b0[8], b1[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const int ul = 4 * t + kq, ulc = ul < kU1 ? ul : kU1 - 1;
                    av[t] = d1own[ul * 16 + n];
                    b0[t] = w1s[ulc * F0P + 16 * wave + n];
                    b1[t] = two ? w1s[ulc * F0P + 16 * (wave + 8) + n] : 0.f;
                }
                __builtin_amdgcn_sched_barrier(0);
                f4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(av[t], b0[t], acc0, 0, 0, 0);
                    if (two) acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(av[t], b1[t], acc1, 0, 0, 0);
                }
                // lane: feature n of the tile, samples 4 kq .. 4 kq + 3
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    xpost(rec + kXB2 + g * 4096 + (4 * kq + r) * 256 + 16 * wave + n, wt.tag, acc0[r]);
                    if (two) xpost(rec + kXB2 + g * 4096 + (4 * kq + r) * 256 + 16 * (wave + 8) + n, wt.tag, acc1[r]);
                }
            }
        }
        // which of the own pooled conv-2 outputs are positive (a0 is overwritten below)
        bool alive2[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int e = tq + kLnThreads * j;
            alive2[j] = e < 4 * F0 && a0[(4 * g + e / F0) * F0P + e % F0] > 0.f;
        }
        __syncthreads();
        // dense 1: w <- w - eta g, U <- U + g on the own rows.  g^T = delta^T a0 on the matrix cores:
        // rows = the own units in two tiles, columns = the F0 inputs in tiles of 16 (tiles w and
        // w + 8 for wave w), contraction over the 16 samples.  A lane ends up with the gradient of
        // the weights (unit 16 mt + 4 kq + r, input 16 nt + n) and keeps their U.
        {
            const int wave = __builtin_amdgcn_readfirstlane(tq >> 6), lane = tq & 63;
            const int n = lane & 15, kq = lane >> 4;
            const int ntile = F0 >> 4;
            if (wave < ntile) {
                const bool two = wave + 8 < ntile;
                float av[2][4], bv[2][4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    av[0][t] = d1own[n * 16 + 4 * t + kq];
                    av[1][t] = d1own[(16 + n) * 16 + 4 * t + kq];
                    bv[0][t] = a0[(4 * t + kq) * F0P + 16 * wave + n];
                    bv[1][t] = two ? a0[(4 * t + kq) * F0P + 16 * (wave + 8) + n] : 0.f;
                }
                __builtin_amdgcn_sched_barrier(0);
                f4 acc[2][2];
#pragma unroll
                for (int nl = 0; nl < 2; ++nl)
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt) acc[nl][mt] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt) {
                        acc[0][mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[mt][t], bv[0][t], acc[0][mt], 0, 0, 0);
                        if (two) acc[1][mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[mt][t], bv[1][t], acc[1][mt], 0, 0, 0);
                    }
#pragma unroll
                for (int nl = 0; nl < 2; ++nl) {
                    if (nl == 1 && !two) break;
                    const int k = 16 * (wave + 8 * nl) + n;
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int ul = 16 * mt + 4 * kq + r;
                            if (ul < kU1) {
                                const float gv = acc[nl][mt][r] * invB;
                                w1s[ul * F0P + k] -= eta * gv;
                                U1[(2 * nl + mt) * 4 + r] += gv;
                            }
                        }
                }
            }
        }
        if (tq < kU1) {
            float s = 0.f;
#pragma unroll
            for (int b = 0; b < kLnB; ++b) s += d1own[tq * 16 + b];
            const float gv = s * invB;
            b1s[tq] -= eta * gv;
            U1b += gv;
        }
        // delta at the own samples' pooled conv-2 outputs (masked by the ReLU): both elements of
        // a thread in one batch of loads
        {
            const u64 *ptr[8];
            bool need[8];
            float val[8];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int e = tq + kLnThreads * j;
                const bool act = e < 4 * F0;
                const int s = act ? e / F0 : 0, f = act ? e % F0 : 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    ptr[4 * j + i] = rec + kXB2 + i * 4096 + (4 * g + s) * 256 + f;
                    need[4 * j + i] = act;
                }
            }
            xfetch<8>(ptr, need, val, wt);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int e = tq + kLnThreads * j;
                if (e < 4 * F0) {
                    float t = val[4 * j];
                    t += val[4 * j + 1];
                    t += val[4 * j + 2];
                    t += val[4 * j + 3];
                    dp2[e] = alive2[j] ? t : 0.f;
                }
            }
        }
        __syncthreads();

        tq = opaque(tq);
        // ---- backward through conv 2 ---------------------------------------------------------------
        // delta at the conv-2 outputs: zero but at the winner of every window
        for (int i = tq; i < 64 * CS2; i += kLnThreads) dc2[i] = 0.f;
        __syncthreads();
        for (int e = tq; e < 4 * F0; e += kLnThreads) {
            const int s = e >> lgF0, f = e & (F0 - 1), c = f / nwin2;
            dc2[(s * 16 + c) * CS2 + pos2[e]] = dp2[e];
        }
        __syncthreads();
        tq = opaque(tq);
        // filter gradient over the own samples on the matrix cores:
        //   gw[c][(ci, ky, kx)] = sum over (sample, position) of delta[c][pos] in[ci][pos + (ky, kx)]
        // rows = the 16 channels, columns = the 150 filter entries of a channel in ten tiles of 16
        // (the last one has 6 idle columns), contraction over the 4 x H2 x H2 positions, four
        // consecutive positions of a map row per step (lane group kq takes position 4 t + kq).  The
        // delta map is zero but at the window winners, which costs nothing here.  Waves 0 and 1
        // take two tiles (one read of the deltas for both).
        {
            const int wave = __builtin_amdgcn_readfirstlane(tq >> 6), lane = tq & 63;
            const int n = lane & 15, kq = lane >> 4;
            const float *abase = dc2 + n * CS2 + kq;
            // where lane group kq sits inside a step: along the row, or (2 x 2 maps) in the map
            const int kqoff = H2 >= 4 ? kq : (kq >> 1) * P1 + (kq & 1);
            const bool two = wave + 8 < 10;
            const float *bbase[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int col = 16 * (wave + (two ? 8 * h : 0)) + n;
                const int cc = col < 150 ? col : 149;     // idle columns read a valid entry
                const int ci = cc / 25, r = cc - 25 * ci, ky = r / 5, kx = r - 5 * ky;
                bbase[h] = p1 + ci * nwin1 + ky * P1 + kx + kqoff;
            }
            f4 acc[2] = {f4{0.f, 0.f, 0.f, 0.f}, f4{0.f, 0.f, 0.f, 0.f}};
            // the steps of one sample: 8 x 8 maps take them eight at a time (four map rows, two steps
            // per row, every offset an immediate), smaller maps one map row (4 x 4) or the whole map
            // (2 x 2) per step
            auto sample_steps = [&](auto twoc, const float *ap, const float *bp0, const float *bp1) {
                constexpr bool TWO = decltype(twoc)::value;
                if (H2 == 8) {
#pragma unroll
                    for (int y0 = 0; y0 < 8; y0 += 4) {
                        float av[8], b0[8], b1[8];
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            const int y = y0 + (i >> 1), x0 = 4 * (i & 1);
                            av[i] = ap[8 * y + x0];
                            b0[i] = bp0[y * P1 + x0];
                            if (TWO) b1[i] = bp1[y * P1 + x0];
                        }
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i], b0[i], acc[0], 0, 0, 0);
                            if (TWO) acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i], b1[i], acc[1], 0, 0, 0);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                } else {
                    const int rows = H2 == 4 ? 4 : 1;
#pragma unroll 1
                    for (int y = 0; y < rows; ++y) {
                        const float a1 = ap[4 * y], c0 = bp0[y * P1];
                        acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, c0, acc[0], 0, 0, 0);
                        if (TWO) acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, bp1[y * P1], acc[1], 0, 0, 0);
                    }
                }
            };
#pragma unroll 1
            for (int sl = 0; sl < 4; ++sl) {
                const float *ap = abase + sl * 16 * CS2, *bp0 = bbase[0] + sl * P1S, *bp1 = bbase[1] + sl * P1S;
                if (two) sample_steps(std::true_type{}, ap, bp0, bp1);
                else sample_steps(std::false_type{}, ap, bp0, bp1);
            }
            // lane: column n of the tile, channels 4 kq .. 4 kq + 3
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int col = 16 * (wave + 8 * h) + n;
                if ((h == 0 || two) && col < 150) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) gsum[156 + (4 * kq + r) * 150 + col] = acc[h][r];
                }
            }
        }
        if (tq >= 480 && tq < 496) {
            const int c = tq - 480;
            float s = 0.f;
            if (nwin2 == 16) {
                f4 v[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) v[i] = *reinterpret_cast<const f4 *>(dp2 + (i >> 2) * F0 + c * 16 + 4 * (i & 3));
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    s += v[i][0];
                    s += v[i][1];
                    s += v[i][2];
                    s += v[i][3];
                }
            } else {
                for (int i = 0; i < 4; ++i)
                    for (int win = 0; win < nwin2; ++win) s += dp2[i * F0 + c * nwin2 + win];
            }
            gsum[2556 + c] = s;
        }
        __syncthreads();
        tq = opaque(tq);
        // the conv-2 part of the filter gradient is complete: post it now, it travels while the
        // rest of the backward pass runs
#pragma unroll
        for (int j = 0; j < 5; ++j) {
            const int e = 156 + tq + kLnThreads * j;
            if (e < kConvP) xpost(rec + kXB3 + g * 2576 + e, wt.tag, gsum[e]);
        }
        // delta at the pooled conv-1 outputs (dense correlation with the flipped filters), masked
        // by the ReLU.
        if constexpr (G28) {
            // On the matrix cores, in two stages.  With the input channel alone as the row index a
            // 16-row tile would hold 6 rows; so the filter column kx joins it:
            //   T[(ci, kx)][s][yy][x'] = sum over (c, ky) of w[c][ci][ky][kx] delta[s][c][yy - ky][x']
            // (30 rows in two tiles; columns = two samples x the 8 positions of a delta row;
            // contraction over the 16 channels, four per step, and the filter rows that reach yy),
            // and then  d[s][ci][yy][xx] = sum over kx of T[(ci, kx)][s][yy][xx - kx],  added in
            // the order of kx through a slice of LDS that belongs to the wave.
            // Work item = output row yy, both sample pairs (one read of the filters for the two
            // column tiles); the rows are dealt so that every wave gets five filter-row passes:
            // {4}, {5}, {6}, {7}, {3, 0}, {8, 11}, {2, 1}, {9, 10}.
            // A step's four lane groups take channels base + 2 kq (base = 0, 1, 8, 9): with the
            // delta maps 68 floats apart their rows then start 8 banks apart.
            __syncthreads();    // gsum has been posted: its space now holds the waves' slices
            const int wave = __builtin_amdgcn_readfirstlane(tq >> 6), lane = tq & 63;
            const int n = lane & 15, kq = lane >> 4;
            const int ya = wave < 4 ? 4 + wave : wave == 4 ? 3 : wave == 5 ? 8 : wave == 6 ? 2 : 9;
            const int yb = wave < 4 ? -1 : wave == 4 ? 0 : wave == 5 ? 11 : wave == 6 ? 1 : 10;
            const int m0 = n, m1 = 16 + n < 30 ? 16 + n : 29;              // rows (ci, kx) of the two tiles
            const float *wa0 = wc2 + 2 * kq * kWS + (m0 / 5) * 25 + m0 % 5;
            const float *wa1 = wc2 + 2 * kq * kWS + (m1 / 5) * 25 + m1 % 5;
            const float *bbase = dc2 + ((n >> 3) * 16 + 2 * kq) * CS2 + (n & 7);   // sample n / 8 of a pair
            float *scr = dpart + wave * kDP;
            // second stage, the same for every item: lane -> three outputs (sample of the pair,
            // input channel, xx); their five addends sit 16 floats apart in the slice
            int rd[3], oo[3];
            uint32_t vm[3];
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const int o = lane + 64 * j, oc = o < 144 ? o : 0;
                const int sl = oc / 72, rem = oc - 72 * sl, ci = rem / 12, xx = rem - 12 * ci;
                rd[j] = ci * 85 + sl * 8 + xx;
                oo[j] = sl * P1S + ci * nwin1 + xx;
                uint32_t m = 0;
#pragma unroll
                for (int kx = 0; kx < 5; ++kx)
                    if (o < 144 && xx - kx >= 0 && xx - kx < 8) m |= 1u << kx;
                vm[j] = m;
            }
#pragma unroll 1
            for (int it = 0; it < 2; ++it) {
                const int yy = it == 0 ? ya : yb;
                if (yy < 0) break;
                const int ky_lo = yy - 7 > 0 ? yy - 7 : 0, ky_hi = yy < 4 ? yy : 4;
                f4 acc[2][2];
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[i >> 1][i & 1] = f4{0.f, 0.f, 0.f, 0.f};
                // operands of one filter row (four steps of four channels); the next row's are
                // fetched before the products of the current one are issued
                auto fetch = [&](int ky, float (&av)[2][4], float (&bv)[2][4]) {
                    const float *ap0 = wa0 + ky * 5, *ap1 = wa1 + ky * 5, *bp = bbase + (yy - ky) * 8;
#pragma unroll
                    for (int tc = 0; tc < 4; ++tc) {
                        const int cb = (tc & 1) + 8 * (tc >> 1);     // 0, 1, 8, 9
                        av[0][tc] = ap0[cb * kWS];
                        av[1][tc] = ap1[cb * kWS];
                        bv[0][tc] = bp[cb * CS2];
                        bv[1][tc] = bp[(32 + cb) * CS2];
                    }
                };
                auto products = [&](const float (&av)[2][4], const float (&bv)[2][4]) {
#pragma unroll
                    for (int tc = 0; tc < 4; ++tc)
#pragma unroll
                        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                            for (int mt = 0; mt < 2; ++mt)
                                acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[mt][tc], bv[nt][tc], acc[nt][mt], 0, 0, 0);
                };
                float xa[2][4], xb[2][4], ya4[2][4], yb4[2][4];
                fetch(ky_lo, xa, xb);
#pragma unroll 1
                for (int ky = ky_lo;; ky += 2) {
                    if (ky + 1 <= ky_hi) fetch(ky + 1, ya4, yb4);
                    __builtin_amdgcn_sched_barrier(0);
                    products(xa, xb);
                    if (ky + 1 > ky_hi) break;
                    if (ky + 2 <= ky_hi) fetch(ky + 2, xa, xb);
                    __builtin_amdgcn_sched_barrier(0);
                    products(ya4, yb4);
                    if (ky + 2 > ky_hi) break;
                }
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) {
                    // lane: column n = (sample of the pair, x'), rows 4 kq + r of both row tiles
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        scr[(4 * kq + r) * 17 + n] = acc[nt][0][r];
                        if (16 + 4 * kq + r < 30) scr[(16 + 4 * kq + r) * 17 + n] = acc[nt][1][r];
                    }
                    // (the wave's LDS operations are carried out in order: no barrier is needed)
                    // (all loads first, then the sums and the stores)
                    float v[3][5], pm[3];
#pragma unroll
                    for (int j = 0; j < 3; ++j) {
#pragma unroll
                        for (int kx = 0; kx < 5; ++kx) v[j][kx] = scr[((vm[j] >> kx) & 1u) ? rd[j] + 16 * kx : 0];
                        pm[j] = p1[oo[j] + 2 * nt * P1S + yy * P1];
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int j = 0; j < 3; ++j) {
                        float t = 0.f;
#pragma unroll
                        for (int kx = 0; kx < 5; ++kx) t += ((vm[j] >> kx) & 1u) ? v[j][kx] : 0.f;
                        if (vm[j]) dp1[oo[j] + 2 * nt * P1S + yy * P1] = pm[j] > 0.f ? t : 0.f;
                    }
                }
            }
        } else {
            // A wave takes one output row yy and two input channels: lane = (channels c
            // and c + 8, sample, input channel); the filter rows that reach row yy are the same
            // for the whole wave (scalar loop bounds), whole delta rows are read without guards, and
            // the eight channel groups of a lane octet are added in a fixed tree.
            const int wave = __builtin_amdgcn_readfirstlane(tq >> 6), lane = tq & 63;
            const int cq = lane & 7, s = (lane >> 3) & 3, cil = lane >> 5;
#pragma unroll 1
            for (int wi = wave; wi < 3 * P1; wi += kLnThreads / 64) {
                const int yy = wi / 3, ci = 2 * (wi - 3 * yy) + cil;
                const int ky_lo = yy - (H2 - 1) > 0 ? yy - (H2 - 1) : 0, ky_hi = yy < 4 ? yy : 4;
                float acc[12];
#pragma unroll
                for (int x = 0; x < 12; ++x) acc[x] = 0.f;
                // operands of one filter row: the delta rows of the lane's two channels and the
                // five weights of each; the next row's operands are fetched before the products
                // of the current one are issued
                auto fetch = [&](int ky, float (&dv)[2][8], float (&wv)[2][5]) {
#pragma unroll
                    for (int cc = 0; cc < 2; ++cc) {
                        const int c = cq + 8 * cc;
                        const float *row = dc2 + (s * 16 + c) * CS2 + (yy - ky) * H2;
                        const float *wrow = wc2 + c * kWS + ci * 25 + ky * 5;
                        if (H2 == 8) {
                            const f4 lo = *reinterpret_cast<const f4 *>(row), hi = *reinterpret_cast<const f4 *>(row + 4);
#pragma unroll
                            for (int x = 0; x < 4; ++x) { dv[cc][x] = lo[x]; dv[cc][4 + x] = hi[x]; }
                        } else {
                            // narrower maps: what lies beyond the row is read (it is inside the
                            // buffer) and dropped
#pragma unroll
                            for (int x = 0; x < 8; ++x) {
                                const float v = row[x];
                                dv[cc][x] = x < H2 ? v : 0.f;
                            }
                        }
#pragma unroll
                        for (int kx = 0; kx < 5; ++kx) wv[cc][kx] = wrow[kx];
                    }
                };
                auto products = [&](const float (&dv)[2][8], const float (&wv)[2][5]) {
#pragma unroll
                    for (int cc = 0; cc < 2; ++cc)
#pragma unroll
                        for (int x = 0; x < 8; ++x)
#pragma unroll
                            for (int kx = 0; kx < 5; ++kx) acc[x + kx] += dv[cc][x] * wv[cc][kx];
                };
                float dva[2][8], wva[2][5], dvb[2][8], wvb[2][5];
                fetch(ky_lo, dva, wva);
                for (int ky = ky_lo;; ky += 2) {
                    if (ky + 1 <= ky_hi) fetch(ky + 1, dvb, wvb);
                    __builtin_amdgcn_sched_barrier(0);
                    products(dva, wva);
                    if (ky + 1 > ky_hi) break;
                    if (ky + 2 <= ky_hi) fetch(ky + 2, dva, wva);
                    __builtin_amdgcn_sched_barrier(0);
                    products(dvb, wvb);
                    if (ky + 2 > ky_hi) break;
                }
                // the eight channel pairs of a lane octet: neighbours, the other pair of the quad,
                // the other quad (fixed order, the same in every run)
#pragma unroll
                for (int x = 0; x < 12; ++x) {
                    float t = acc[x];
                    t += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, t), 0xB1, 0xF, 0xF, true));
                    t += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, t), 0x4E, 0xF, 0xF, true));
                    t += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, t), 0x141, 0xF, 0xF, true));
                    acc[x] = t;
                }
                if (cq == 0) {
#pragma unroll
                    for (int x = 0; x < 12; ++x)
                        if (x < P1) {
                            const int o = s * P1S + ci * nwin1 + yy * P1 + x;
                            dp1[o] = p1[o] > 0.f ? acc[x] : 0.f;
                        }
                }
            }
        }
        __syncthreads();

        tq = opaque(tq);
        // the four partial conv-2 gradients were posted before the last phase: ask for them now, the
        // words are looked at after the conv-1 gradient below (thread: elements 156 + tq + 512 j)
        u64 early[5][4];
#pragma unroll
        for (int j = 0; j < 5; ++j) {
            const int e = 156 + tq + kLnThreads * j;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                early[j][i] = __hip_atomic_load(rec + kXB3 + i * 2576 + (e < kConvP ? e : 156), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        // ---- conv-1 filter gradient over the own samples: thread = (window group, channel,
        // filter row); one position per window; the bias gradient is the sum of the deltas the
        // thread of filter row 0 reads anyway ------------------------------------------------------
        if (tq < 14 * 36) {
            const int grp = tq / 36, r = tq % 36;
            if (r < 30) {
                const int c = r / 5, ky = r % 5;
                float acc[5] = {0.f, 0.f, 0.f, 0.f, 0.f};
                float bsum = 0.f;    // the deltas themselves: the bias gradient (kept by the ky = 0 thread)
#pragma unroll 1
                for (int s = 0; s < 4; ++s) {
                    const float *dl_p = dp1 + s * P1S + c * nwin1;
                    const uint16_t *of_p = off1 + (s * 6 + c) * nwin1;
                    const float *base = xs + s * npix + ky * H0;
#pragma unroll 1
                    for (int w0 = grp; w0 < nwin1; w0 += 4 * 14) {
                        float dl[4], rv[4][5];
                        int of[4];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int win = w0 + 14 * i < nwin1 ? w0 + 14 * i : w0;
                            dl[i] = dl_p[win];
                            of[i] = of_p[win];
                        }
#pragma unroll
                        for (int i = 0; i < 4; ++i)
#pragma unroll
                            for (int kx = 0; kx < 5; ++kx) rv[i][kx] = base[of[i] + kx];
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float dv = w0 + 14 * i < nwin1 ? dl[i] : 0.f;
                            bsum += dv;
#pragma unroll
                            for (int kx = 0; kx < 5; ++kx) acc[kx] += dv * rv[i][kx];
                        }
                    }
                }
#pragma unroll
                for (int kx = 0; kx < 5; ++kx) c1part[grp * 160 + c * 25 + ky * 5 + kx] = acc[kx];
                if (ky == 0) c1part[grp * 160 + 150 + c] = bsum;
            }
        }
        __syncthreads();
        // ---- filter banks: exchange the partial gradients, add them in workgroup order, update ----
        if (tq < 156) {   // the conv-1 part: the thread that adds the window groups posts the sum
            float s = 0.f;
#pragma unroll
            for (int grp = 0; grp < 14; ++grp) s += c1part[grp * 160 + tq];
            xpost(rec + kXB3 + g * 2576 + tq, wt.tag, s);
        }
        // the next recursion's rows and labels (xs and labs are not read any more)
        if (more) store_rows(xr, labr);
        {   // the conv-1 part: threads 0 .. 155
            const bool act = tq < 156;
            const u64 *ptr[4];
            bool need[4];
            float val[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ptr[i] = rec + kXB3 + i * 2576 + (act ? tq : 0);
                need[i] = act;
            }
            xfetch<4>(ptr, need, val, wt);
            if (act) {
                float t = val[0];
                t += val[1];
                t += val[2];
                t += val[3];
                const float gv = t * invB;
                wc1[tq] -= eta * gv;
                UC[0] += gv;
            }
        }
#pragma unroll
        for (int j = 0; j < 5; ++j) {   // the conv-2 part and its biases: the words asked for earlier
            const int e = 156 + tq + kLnThreads * j;
            const bool act = e < kConvP;
            float val[4];
            bool ok = true;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ok = ok && (uint32_t)(early[j][i] >> 32) == wt.tag;
                val[i] = __uint_as_float((uint32_t)early[j][i]);
            }
            if (act && !ok) {   // not there yet when asked: fetch again (rare)
                const u64 *ptr[4];
                bool need[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    ptr[i] = rec + kXB3 + i * 2576 + e;
                    need[i] = true;
                }
                xfetch<4>(ptr, need, val, wt);
            }
            if (act) {
                float t = val[0];
                t += val[1];
                t += val[2];
                t += val[3];
                const float gv = t * invB;
                float *w = e < 2556 ? wc2 + ((e - 156) / 150) * kWS + (e - 156) % 150 : wc2b + (e - 2556);
                *w -= eta * gv;
                UC[1 + j] += gv;
            }
        }
        __syncthreads();
    }

    // ---- end of round: the replica and the message payload go to HBM ------------------------------
    {   // dense 1 in the ownership of its update: lane (n, kq) of wave w, input tiles w and w + 8
        const int wave = tid >> 6, n = tid & 15, kq = (tid & 63) >> 4, ntile = F0 >> 4;
#pragma unroll
        for (int nl = 0; nl < 2; ++nl) {
            const int nt = wave + 8 * nl;
            if (nt < ntile) {
                const int k = 16 * nt + n;
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int ul = 16 * mt + 4 * kq + r;
                        if (ul < kU1) {
                            const int64_t o = d.o_f1 + (int64_t)(kU1 * g + ul) * F0 + k;
                            Wc[o] = w1s[ul * F0P + k];
                            Uc[o] = U1[(2 * nl + mt) * 4 + r];
                        }
                    }
            }
        }
    }
    if (tid < kU1) {
        const int64_t o = d.o_f1 + (int64_t)kF1 * F0 + kU1 * g + tid;
        Wc[o] = b1s[tid];
        Uc[o] = U1b;
    }
    {   // dense 2 in the ownership of its update
        const int wave = tid >> 6, n = tid & 15, kq = (tid & 63) >> 4, k = 16 * wave + n;
        if (k < kF1) {
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int ul = 16 * mt + 4 * kq + r;
                    if (ul < kU2) {
                        const int64_t o = d.o_f2 + (int64_t)(kU2 * g + ul) * kF1 + k;
                        Wc[o] = w2s[ul * kS1 + k];
                        Uc[o] = U2[4 * mt + r];
                    }
                }
        }
    }
    if (tid < kU2) {
        const int64_t o = d.o_f2 + kF2 * kF1 + kU2 * g + tid;
        Wc[o] = b2s[tid];
        Uc[o] = U2b;
    }
    if (g == 0) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int e = tid + kLnThreads * j;
            if (e < kNC * kF2) {
                Wc[d.o_f3 + e] = w3s[(e / kF2) * kS2 + e % kF2];
                Uc[d.o_f3 + e] = U3[j];
            }
        }
        if (tid < kNC) {
            Wc[d.o_f3 + kNC * kF2 + tid] = b3s[tid];
            Uc[d.o_f3 + kNC * kF2 + tid] = U3b;
        }
        if (tid < 156) {   // the filter banks in the ownership of their update
            Wc[tid] = wc1[tid];
            Uc[tid] = UC[0];
        }
#pragma unroll
        for (int j = 0; j < 5; ++j) {
            const int e = 156 + tid + kLnThreads * j;
            if (e < kConvP) {
                Wc[e] = e < 2556 ? wc2[((e - 156) / 150) * kWS + (e - 156) % 150] : wc2b[e - 2556];
                Uc[e] = UC[1 + j];
            }
        }
        if (tid == 0) *as_global(p.loss) = lossacc[0];
    }
}

__global__ void k_zero_words_ln(u64 *p, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0ull;
}

bool lenet_dims(const LayerGeom *lay, int L, int B, LenetDims *d) {
    if (L != 7 || B != kLnB) return false;
    const LayerGeom &c1 = lay[0], &q1 = lay[1], &c2 = lay[2], &q2 = lay[3], &f1 = lay[4], &f2 = lay[5], &f3 = lay[6];
    if (c1.type != 0 || q1.type != 1 || c2.type != 0 || q2.type != 1 || f1.type != 2 || f2.type != 2 || f3.type != 2) return false;
    if (c1.k != 5 || c1.pad != 0 || !c1.relu || c1.ic != 1 || c1.oc != 6 || c1.ih != c1.iw) return false;
    if (c2.k != 5 || c2.pad != 0 || !c2.relu || c2.oc != 16) return false;
    if (f1.oc != kF1 || !f1.relu || f2.oc != kF2 || !f2.relu || f3.oc != kNC || f3.relu) return false;
    d->H0 = c1.ih; d->P1 = q1.oh; d->H2 = c2.oh; d->P2 = q2.oh;
    d->F0 = 16 * d->P2 * d->P2;
    if (d->H0 > 32 || (d->H0 * d->H0) % 4 || d->P1 > 12 || (d->P1 & 1) || d->H2 > 8) return false;
    if (d->F0 != 16 && d->F0 != 64 && d->F0 != 256) return false;   // P2 = 1, 2 or 4
    d->lgF0 = d->F0 == 16 ? 4 : d->F0 == 64 ? 6 : 8;
    if ((int64_t)d->F0 != f1.in_size) return false;
    d->o_f1 = f1.w_off; d->o_f2 = f2.w_off; d->o_f3 = f3.w_off;
    if (c1.w_off != 0 || c1.b_off != 150 || c2.w_off != 156 || c2.b_off != 2556 || f1.w_off != kConvP) return false;
    return true;
}

size_t lenet_lds_bytes(const LenetDims &d) {
    auto up4 = [](int n) { return (n + 3) & ~3; };
    const int nwin1 = d.P1 * d.P1, P1S = 6 * nwin1 + 8, F0P = d.F0 + 4;
    size_t fl = up4(4 * d.H0 * d.H0) + 4 * P1S + 16 * F0P;
    fl += (2 * up4(4 * 6 * nwin1) + 2 * up4(4 * d.F0) + up4(4 * d.F0)) / 4;
    fl += 160 + 16 * kWS + 16 + kU1 * F0P + 32 + kU2 * kS1 + 32 + kNC * kS2 + 16;
    fl += 16 * kS1 + 16 * kS2 + 256 + 16 * kS2 + 16 * 24 + 16 * 32 + up4(4 * d.F0) + 2576 + 14 * 160 + 16 + 16 + 4;
    return fl * 4;
}

int g_lenet_per_cu[2] = {0, 0};

}  // namespace

bool lenet_round_supported(const LayerGeom *lay, int L, int B) {
    LenetDims d;
    if (!lenet_dims(lay, L, B, &d)) return false;
    // the regions that take turns in LDS must fit where they are put
    const int P1S = 6 * d.P1 * d.P1 + 8;
    if (64 * (d.H2 * d.H2 + 4) > 16 * (d.F0 + 4) + 16 * 24 + 16 * 32) return false;   // d conv-2 outputs over a0 .. d1own
    if (4 * P1S > 16 * kS1 + 16 * kS2 + 256 + 16 * kS2) return false;     // d pooled conv-1 outputs over h1 .. dh2
    return lenet_lds_bytes(d) <= 160 * 1024;
}

size_t lenet_round_scratch_bytes(int n_clients) { return (size_t)n_clients * kXWords * 8 + 256; }

hipError_t lenet_clear_error_flag(hipStream_t s, void *scratch, int n_clients) {
    u64 *xrec = static_cast<u64 *>(scratch);
    k_zero_words_ln<<<1, 64, 0, s>>>(xrec + (size_t)n_clients * kXWords, 1);
    return hipGetLastError();
}

const int *lenet_error_flag_ptr(void *scratch, int n_clients) {
    return reinterpret_cast<const int *>(static_cast<u64 *>(scratch) + (size_t)n_clients * kXWords);
}

hipError_t launch_lenet_round(hipStream_t s, Profiler *prof, const RoundParams *dp, int nact, int max_m,
                              const float *Wg, const LayerGeom *lay, int L, int B, void *scratch,
                              int n_clients, uint32_t *epoch) {
    if (nact <= 0) return hipSuccess;
    LenetDims d;
    if (!lenet_dims(lay, L, B, &d)) return hipErrorInvalidValue;
    const size_t lds = lenet_lds_bytes(d);
    hipError_t e;
    const bool g28 = d.H0 == 28 && d.P1 == 12 && d.H2 == 8 && d.P2 == 4 && d.F0 == 256 && d.lgF0 == 8;
    const void *fn = g28 ? reinterpret_cast<const void *>(k_lenet_round<true>) : reinterpret_cast<const void *>(k_lenet_round<false>);
    if (g_lenet_per_cu[g28] == 0) {
        e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
    }
    int dev = 0, cus = 0, per_cu = 0;
    e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    e = g28 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_lenet_round<true>, kLnThreads, lds)
            : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_lenet_round<false>, kLnThreads, lds);
    if (e != hipSuccess) return e;
    g_lenet_per_cu[g28] = per_cu;
    // clusters per launch: every workgroup that polls must be resident together with its peers
    const int per_launch = cus * per_cu / kLnG;
    if (per_launch < 1) return hipErrorLaunchOutOfResources;
    u64 *xrec = static_cast<u64 *>(scratch);
    int *errflag = reinterpret_cast<int *>(xrec + (size_t)n_clients * kXWords);
    // step tags of this launch: never 0 (the cleared state) and never a tag that an earlier
    // launch may have left in the records
    if (*epoch == 0 || *epoch > 0xFFFFFFFFu - (uint32_t)max_m - 2u) {
        const size_t words = (size_t)n_clients * kXWords;
        k_zero_words_ln<<<(unsigned)((words + 255) / 256), 256, 0, s>>>(xrec, words);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        *epoch = 1;
    }
    const uint32_t tag0 = *epoch;
    *epoch += (uint32_t)max_m + 1u;
    for (int a0 = 0; a0 < nact; a0 += per_launch) {
        const int here = nact - a0 < per_launch ? nact - a0 : per_launch;
        const unsigned grid = (unsigned)(8 * ((here + 7) / 8) * kLnG);
        if (prof && prof->on[F_LENET_ROUND]) prof->before(F_LENET_ROUND, s);
        if (g28) k_lenet_round<true><<<grid, kLnThreads, lds, s>>>(dp + a0, here, a0, Wg, d, xrec, tag0, errflag);
        else k_lenet_round<false><<<grid, kLnThreads, lds, s>>>(dp + a0, here, a0, Wg, d, xrec, tag0, errflag);
        if (prof && prof->on[F_LENET_ROUND]) prof->after(F_LENET_ROUND, s);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace aet
