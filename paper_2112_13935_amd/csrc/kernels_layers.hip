// Layer-by-layer engine: one SGD recursion of every active client as a short sequence of
// kernels, each batched over the clients (blockIdx.z) and the mini-batch.  It runs any
// model the ABI can describe; the fused persistent kernels for single-dense and
// dense-ReLU-dense models take over for those shapes.
//
// One recursion (Algorithm 2, MainComputeNode, body of the while loop), for client c:
//   draw B sample indices and gather the rows      -> k_gather
//   forward pass, layer by layer                   -> k_conv_fwd / k_pool_fwd / k_dense_fwd
//   softmax cross-entropy, d loss / d logits       -> k_softmax_ce
//   backward pass; each parameter layer first hands the gradient to the layer below
//   (k_*_bwd_data, which reads the not-yet-updated weights) and then forms its own
//   gradient g and applies  w <- w - eta g,  U <- U + g  in the same kernel
//   (k_*_bwd_weight), so g never goes to memory.
// Clients whose round has fewer recursions than the step counter simply exit.
#include "aet_device.h"
#include "aet_internal.h"

namespace aet {

// time the launch if its family is being profiled
#define AET_TIMED(fam, ...)                              \
    do {                                                 \
        if (prof && prof->on[fam]) prof->before(fam, s); \
        __VA_ARGS__;                                     \
        if (prof && prof->on[fam]) prof->after(fam, s);  \
    } while (0)

#define AET_RETURN_IF(e)                 \
    do {                                 \
        hipError_t e__ = (e);            \
        if (e__ != hipSuccess) return e__; \
    } while (0)

__global__ void k_begin_round(const RoundParams *__restrict__ rp, const float *__restrict__ Wg,
                              int64_t P) {
    const RoundParams p = rp[blockIdx.y];
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < P) {
        if (Wg) p.W[i] = Wg[i];  // adopt the broadcast global model (server form)
        p.U[i] = 0.f;
    }
    if (i == 0) *p.loss = 0.f;
}

// act0[a][b][:] = X_c[row(q0 + u*B + b)][:]
__global__ void k_gather(const RoundParams *__restrict__ rp, int u, int B, int D,
                         float *__restrict__ act0, int32_t *__restrict__ labels) {
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    const int b = blockIdx.y;
    const uint32_t row = sample_row(p.key, (uint64_t)(p.q0 + (int64_t)u * B + b), p.n_samples);
    const int d = blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t o = ((int64_t)blockIdx.z * B + b);
    if (d < D) act0[o * D + d] = p.X[(int64_t)row * D + d];
    if (d == 0) labels[o] = p.y[row];
}

// out[a][b][o] = relu?(bias[o] + sum_k W[o][k] in[a][b][k]); one wave per output feature
__global__ void __launch_bounds__(256)
k_dense_fwd(const RoundParams *__restrict__ rp, int u, int B, int K, int O, int64_t w_off,
            int64_t b_off, int relu, const float *__restrict__ in, float *__restrict__ out) {
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int o = blockIdx.x * 4 + wave;
    if (o >= O) return;
    const float *w = p.W + w_off + (int64_t)o * K;
    const float bias = p.W[b_off + o];
    const float *inb = in + (int64_t)blockIdx.z * B * K;
    float *outb = out + (int64_t)blockIdx.z * B * O;
    for (int b = 0; b < B; ++b) {
        float s = 0.f;
        for (int k = lane; k < K; k += 64) s += w[k] * inb[(int64_t)b * K + k];
        s = wave_sum(s) + bias;
        if (relu && !(s > 0.f)) s = 0.f;
        if (lane == 0) outb[(int64_t)b * O + o] = s;
    }
}

// din[a][b][k] = sum_o W[o][k] dout[a][b][o], masked by the ReLU of the layer below
__global__ void __launch_bounds__(256)
k_dense_bwd_data(const RoundParams *__restrict__ rp, int u, int B, int K, int O, int64_t w_off,
                 const float *__restrict__ dout, float *__restrict__ din,
                 const float *__restrict__ mask_src) {
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K) return;
    const int b = blockIdx.y;
    const float *w = p.W + w_off;
    const float *d = dout + ((int64_t)blockIdx.z * B + b) * O;
    float s = 0.f;
    for (int o = 0; o < O; ++o) s += w[(int64_t)o * K + k] * d[o];
    const int64_t i = ((int64_t)blockIdx.z * B + b) * K + k;
    if (mask_src && !(mask_src[i] > 0.f)) s = 0.f;
    din[i] = s;
}

// g[o][k] = (1/B) sum_b dout[b][o] in[b][k];  W -= eta g;  U += g   (and the bias)
__global__ void __launch_bounds__(256)
k_dense_bwd_weight(const RoundParams *__restrict__ rp, int u, int B, int K, int O, int64_t w_off,
                   int64_t b_off, const float *__restrict__ in, const float *__restrict__ dout) {
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K) return;
    const int o = blockIdx.y;
    const float *inb = in + (int64_t)blockIdx.z * B * K;
    const float *d = dout + (int64_t)blockIdx.z * B * O;
    const float invB = 1.0f / (float)B;
    float g = 0.f, gb = 0.f;
    for (int b = 0; b < B; ++b) {
        const float dv = d[(int64_t)b * O + o];
        g += dv * inb[(int64_t)b * K + k];
        gb += dv;
    }
    g *= invB;
    const int64_t wi = w_off + (int64_t)o * K + k;
    p.W[wi] -= p.eta * g;
    p.U[wi] += g;
    if (k == 0) {
        gb *= invB;
        p.W[b_off + o] -= p.eta * gb;
        p.U[b_off + o] += gb;
    }
}

template <int KS>
__global__ void __launch_bounds__(256)
k_conv_fwd(const RoundParams *__restrict__ rp, int u, int B, LayerGeom g,
           const float *__restrict__ in, float *__restrict__ out) {
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= g.oc * g.oh * g.ow) return;
    const int ox = idx % g.ow, oy = (idx / g.ow) % g.oh, co = idx / (g.ow * g.oh);
    const int64_t sample = (int64_t)blockIdx.z * B + blockIdx.y;
    const float *x = in + sample * g.in_size;
    const float *w = p.W + g.w_off + (int64_t)co * g.ic * KS * KS;
    float s = p.W[g.b_off + co];
    for (int ci = 0; ci < g.ic; ++ci) {
#pragma unroll
        for (int ky = 0; ky < KS; ++ky) {
            const int iy = oy + ky - g.pad;
            if (iy < 0 || iy >= g.ih) continue;
#pragma unroll
            for (int kx = 0; kx < KS; ++kx) {
                const int ix = ox + kx - g.pad;
                if (ix < 0 || ix >= g.iw) continue;
                s += w[(ci * KS + ky) * KS + kx] * x[((int64_t)ci * g.ih + iy) * g.iw + ix];
            }
        }
    }
    if (g.relu && !(s > 0.f)) s = 0.f;
    out[sample * g.out_size + idx] = s;
}

// din[ci][iy][ix] = sum_{co,ky,kx} W[co][ci][ky][kx] dout[co][iy-ky+pad][ix-kx+pad]
template <int KS>
__global__ void __launch_bounds__(256)
k_conv_bwd_data(const RoundParams *__restrict__ rp, int u, int B, LayerGeom g,
                const float *__restrict__ dout, float *__restrict__ din,
                const float *__restrict__ mask_src) {
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= g.ic * g.ih * g.iw) return;
    const int ix = idx % g.iw, iy = (idx / g.iw) % g.ih, ci = idx / (g.iw * g.ih);
    const int64_t sample = (int64_t)blockIdx.z * B + blockIdx.y;
    const float *d = dout + sample * g.out_size;
    const float *w = p.W + g.w_off;
    float s = 0.f;
    for (int co = 0; co < g.oc; ++co) {
#pragma unroll
        for (int ky = 0; ky < KS; ++ky) {
            const int oy = iy - ky + g.pad;
            if (oy < 0 || oy >= g.oh) continue;
#pragma unroll
            for (int kx = 0; kx < KS; ++kx) {
                const int ox = ix - kx + g.pad;
                if (ox < 0 || ox >= g.ow) continue;
                s += w[(((int64_t)co * g.ic + ci) * KS + ky) * KS + kx] *
                     d[((int64_t)co * g.oh + oy) * g.ow + ox];
            }
        }
    }
    const int64_t i = sample * g.in_size + idx;
    if (mask_src && !(mask_src[i] > 0.f)) s = 0.f;
    din[i] = s;
}

// One block per (cin, cout) filter plane: g[ky][kx] = (1/B) sum_{b,oy,ox} dout * in, then
// the fused update.  The cin == 0 block also does the bias of its output channel.
template <int KS>
__global__ void __launch_bounds__(256)
k_conv_bwd_weight(const RoundParams *__restrict__ rp, int u, int B, LayerGeom g,
                  const float *__restrict__ in, const float *__restrict__ dout) {
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    const int ci = blockIdx.x, co = blockIdx.y;
    constexpr int NA = KS * KS + 1;
    float acc[NA];
#pragma unroll
    for (int j = 0; j < NA; ++j) acc[j] = 0.f;
    const int plane = g.oh * g.ow;
    const int total = B * plane;
    const float *inb = in + (int64_t)blockIdx.z * B * g.in_size + (int64_t)ci * g.ih * g.iw;
    const float *db = dout + (int64_t)blockIdx.z * B * g.out_size + (int64_t)co * plane;
    for (int t = threadIdx.x; t < total; t += blockDim.x) {
        const int b = t / plane, r = t - b * plane;
        const int oy = r / g.ow, ox = r - oy * g.ow;
        const float d = db[(int64_t)b * g.out_size + r];
        const float *x = inb + (int64_t)b * g.in_size;
        acc[KS * KS] += d;
#pragma unroll
        for (int ky = 0; ky < KS; ++ky) {
            const int iy = oy + ky - g.pad;
            if (iy < 0 || iy >= g.ih) continue;
#pragma unroll
            for (int kx = 0; kx < KS; ++kx) {
                const int ix = ox + kx - g.pad;
                if (ix < 0 || ix >= g.iw) continue;
                acc[ky * KS + kx] += d * x[iy * g.iw + ix];
            }
        }
    }
    __shared__ float red[4][NA];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int j = 0; j < NA; ++j) {
        const float v = wave_sum(acc[j]);
        if (lane == 0) red[wave][j] = v;
    }
    __syncthreads();
    if (threadIdx.x < NA) {
        const int j = threadIdx.x;
        const float gsum = (red[0][j] + red[1][j] + red[2][j] + red[3][j]) * (1.0f / (float)B);
        if (j < KS * KS) {
            const int64_t wi = g.w_off + ((int64_t)co * g.ic + ci) * KS * KS + j;
            p.W[wi] -= p.eta * gsum;
            p.U[wi] += gsum;
        } else if (ci == 0) {
            p.W[g.b_off + co] -= p.eta * gsum;
            p.U[g.b_off + co] += gsum;
        }
    }
}

// 2x2 / stride 2 max pooling; the first maximum in row-major window order wins
__global__ void __launch_bounds__(256)
k_pool_fwd(const RoundParams *__restrict__ rp, int u, int B, LayerGeom g,
           const float *__restrict__ in, float *__restrict__ out, uint8_t *__restrict__ amax) {
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= g.oc * g.oh * g.ow) return;
    const int ox = idx % g.ow, oy = (idx / g.ow) % g.oh, c = idx / (g.ow * g.oh);
    const int64_t sample = (int64_t)blockIdx.z * B + blockIdx.y;
    const float *x = in + sample * g.in_size + ((int64_t)c * g.ih + 2 * oy) * g.iw + 2 * ox;
    float best = x[0];
    int which = 0;
    if (x[1] > best) { best = x[1]; which = 1; }
    if (x[g.iw] > best) { best = x[g.iw]; which = 2; }
    if (x[g.iw + 1] > best) { best = x[g.iw + 1]; which = 3; }
    out[sample * g.out_size + idx] = best;
    amax[sample * g.out_size + idx] = (uint8_t)which;
}

__global__ void __launch_bounds__(256)
k_pool_bwd(const RoundParams *__restrict__ rp, int u, int B, LayerGeom g,
           const float *__restrict__ dout, const uint8_t *__restrict__ amax,
           float *__restrict__ din, const float *__restrict__ mask_src) {
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= g.oc * g.oh * g.ow) return;
    const int ox = idx % g.ow, oy = (idx / g.ow) % g.oh, c = idx / (g.ow * g.oh);
    const int64_t sample = (int64_t)blockIdx.z * B + blockIdx.y;
    const float d = dout[sample * g.out_size + idx];
    const int which = amax[sample * g.out_size + idx];
    const int64_t base = sample * g.in_size + ((int64_t)c * g.ih + 2 * oy) * g.iw + 2 * ox;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t i = base + (j >> 1) * g.iw + (j & 1);
        float v = (j == which) ? d : 0.f;
        if (mask_src && !(mask_src[i] > 0.f)) v = 0.f;
        din[i] = v;
    }
}

// The same two kernels for layers whose input rows are 16-byte aligned (input width a
// multiple of 4): a thread owns two neighbouring windows, reads and writes float4 rows.
typedef float pf4 __attribute__((ext_vector_type(4)));
typedef float pf2 __attribute__((ext_vector_type(2)));

__global__ void __launch_bounds__(256)
k_pool_fwd_pair(const RoundParams *__restrict__ rp, int u, int B, LayerGeom g,
                const float *__restrict__ in, float *__restrict__ out, uint8_t *__restrict__ amax) {
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;   // pair of outputs 2 idx, 2 idx + 1
    const int owh = g.ow >> 1;
    if (idx >= g.oc * g.oh * owh) return;
    const int oxp = idx % owh, oy = (idx / owh) % g.oh, c = idx / (owh * g.oh);
    const int64_t sample = (int64_t)blockIdx.z * B + blockIdx.y;
    const float *x = in + sample * g.in_size + ((int64_t)c * g.ih + 2 * oy) * g.iw + 4 * oxp;
    const pf4 r0 = *reinterpret_cast<const pf4 *>(x), r1 = *reinterpret_cast<const pf4 *>(x + g.iw);
    pf2 best;
    unsigned which2 = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        float b = r0[2 * h];
        unsigned w = 0;
        if (r0[2 * h + 1] > b) { b = r0[2 * h + 1]; w = 1; }
        if (r1[2 * h] > b) { b = r1[2 * h]; w = 2; }
        if (r1[2 * h + 1] > b) { b = r1[2 * h + 1]; w = 3; }
        best[h] = b;
        which2 |= w << (8 * h);
    }
    const int64_t o = sample * g.out_size + 2 * (int64_t)idx;
    *reinterpret_cast<pf2 *>(out + o) = best;
    *reinterpret_cast<uint16_t *>(amax + o) = (uint16_t)which2;
}

__global__ void __launch_bounds__(256)
k_pool_bwd_pair(const RoundParams *__restrict__ rp, int u, int B, LayerGeom g,
                const float *__restrict__ dout, const uint8_t *__restrict__ amax,
                float *__restrict__ din, const float *__restrict__ mask_src) {
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    const int owh = g.ow >> 1;
    if (idx >= g.oc * g.oh * owh) return;
    const int oxp = idx % owh, oy = (idx / owh) % g.oh, c = idx / (owh * g.oh);
    const int64_t sample = (int64_t)blockIdx.z * B + blockIdx.y;
    const int64_t o = sample * g.out_size + 2 * (int64_t)idx;
    const pf2 d = *reinterpret_cast<const pf2 *>(dout + o);
    const unsigned which2 = *reinterpret_cast<const uint16_t *>(amax + o);
    const int64_t base = sample * g.in_size + ((int64_t)c * g.ih + 2 * oy) * g.iw + 4 * oxp;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        pf4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int h = e >> 1, j = 2 * r + (e & 1);
            v[e] = ((which2 >> (8 * h)) & 0xffu) == (unsigned)j ? d[h] : 0.f;
        }
        const int64_t i = base + (int64_t)r * g.iw;
        if (mask_src) {
            const pf4 k = *reinterpret_cast<const pf4 *>(mask_src + i);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (!(k[e] > 0.f)) v[e] = 0.f;
        }
        *reinterpret_cast<pf4 *>(din + i) = v;
    }
}

// rows of the pooling input are 16-byte aligned and the windows come in pairs
static bool pool_pairs(const LayerGeom &g) {
    return (g.iw & 3) == 0 && (g.ow & 1) == 0 && 2 * g.ow == g.iw && 2 * g.oh <= g.ih;
}

// loss and d loss / d logits of the mini-batch; one block per client
__global__ void __launch_bounds__(256)
k_softmax_ce(const RoundParams *__restrict__ rp, int u, int B, int C,
             const float *__restrict__ logits, const int32_t *__restrict__ labels,
             float *__restrict__ dz) {
    const RoundParams p = rp[blockIdx.x];
    if (u >= p.m) return;
    __shared__ float sl[256];
    const int b = threadIdx.x;
    float loss = 0.f;
    if (b < B) {
        const float *z = logits + ((int64_t)blockIdx.x * B + b) * C;
        float *d = dz + ((int64_t)blockIdx.x * B + b) * C;
        const int lab = labels[(int64_t)blockIdx.x * B + b];
        if (C <= 16) {
            // the row in registers: its loads travel together (one trip to memory, not C)
            float zv[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) zv[j] = z[j < C ? j : 0];
            float zmax = zv[0];
#pragma unroll
            for (int j = 1; j < 16; ++j)
                if (j < C) zmax = fmaxf(zmax, zv[j]);
            float sum = 0.f;
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (j < C) sum += expf(zv[j] - zmax);
            const float lse = zmax + logf(sum);
            float zl = zv[0];
#pragma unroll
            for (int j = 1; j < 16; ++j)
                if (j == lab) zl = zv[j];
            loss = lse - zl;
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (j < C) d[j] = expf(zv[j] - lse) - (j == lab ? 1.f : 0.f);
        } else {
            float zmax = z[0];
            for (int j = 1; j < C; ++j) zmax = fmaxf(zmax, z[j]);
            float sum = 0.f;
            for (int j = 0; j < C; ++j) sum += expf(z[j] - zmax);
            const float lse = zmax + logf(sum);
            loss = lse - z[lab];
            for (int j = 0; j < C; ++j) d[j] = expf(z[j] - lse) - (j == lab ? 1.f : 0.f);
        }
    }
    sl[b] = loss;
    __syncthreads();
    if (b == 0) {
        float s = 0.f;
        for (int j = 0; j < B; ++j) s += sl[j];
        *p.loss += s / (float)B;
    }
}

hipError_t launch_begin_round(hipStream_t s, Profiler *prof, const RoundParams *dp, int nact,
                              const float *Wg, int64_t P) {
    if (nact <= 0) return hipSuccess;
    dim3 grid((unsigned)((P + 255) / 256), (unsigned)nact);
    AET_TIMED(F_BEGIN_ROUND, k_begin_round<<<grid, 256, 0, s>>>(dp, Wg, P));
    return hipGetLastError();
}

template <int KS>
static hipError_t conv_step(hipStream_t s, Profiler *prof, const RoundParams *dp, int nact, int u, int B,
                            const LayerGeom &g, int which, const float *a, const float *b,
                            float *c, const float *mask) {
    if (which == 0) {
        dim3 grid((unsigned)((g.out_size + 255) / 256), B, nact);
        AET_TIMED(F_CONV_FWD, k_conv_fwd<KS><<<grid, 256, 0, s>>>(dp, u, B, g, a, c));
    } else if (which == 1) {
        dim3 grid((unsigned)((g.in_size + 255) / 256), B, nact);
        AET_TIMED(F_CONV_BWD_DATA, k_conv_bwd_data<KS><<<grid, 256, 0, s>>>(dp, u, B, g, a, c, mask));
    } else {
        dim3 grid(g.ic, g.oc, nact);
        AET_TIMED(F_CONV_BWD_WEIGHT, k_conv_bwd_weight<KS><<<grid, 256, 0, s>>>(dp, u, B, g, a, b));
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Backward-weight of a convolution with very few channels (LeNet's first layer: 1 -> 6),
// where 16 x 16 matrix tiles would be mostly padding: plain FMAs, one workgroup per
// (client, output channel, input channel).  A thread owns one filter row ky and one output
// row y of one of the samples in flight; it slides along the row with the KS input values
// of the window in registers (one new input value and one d(output) value per pixel feed KS
// FMAs).  The per-row sums are added in fixed order (sample slot, then y), scaled by 1/B and
// applied:  w <- w - eta g,  U <- U + g.  Stride 1, zero padding.
// ---------------------------------------------------------------------------------------
constexpr int kDirectPos = 4;   // tile positions one thread stages, at most
constexpr int kDirectSlots = 4; // samples in flight, at most

template <int KS>
__global__ void __launch_bounds__(256)
k_conv_wgrad_direct(const RoundParams *__restrict__ rp, int u, int B, LayerGeom g,
                    const float *__restrict__ in, const float *__restrict__ dout) {
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    const int oc = blockIdx.x, ic = blockIdx.y, tid = threadIdx.x;
    const int IWP = (g.iw + 2 * g.pad) | 1, IHP = g.ih + 2 * g.pad;   // padded plane, odd row stride
    const int OWS = g.ow | 1;
    const int rows = KS * g.oh;              // threads per sample in flight
    const int SPW = 256 / rows < kDirectSlots ? 256 / rows : kDirectSlots;   // samples in flight
    const int iplane = IHP * IWP, dplane = g.oh * OWS;
    const int ihw = g.ih * g.iw, ohw = g.oh * g.ow;
    extern __shared__ float sm[];
    float *Ism = sm;                         // [SPW][IHP][IWP], borders zero
    float *Dsm = Ism + SPW * iplane;         // [SPW][oh][OWS]
    float *red = Dsm + SPW * dplane;         // [SPW * rows][KS + 1]: row sums per kx, and of d(output)
    const int slot = tid / rows, rem = tid - slot * rows;
    const int ky = rem / g.oh, y = rem - ky * g.oh;
    const bool active = slot < SPW;
    const int64_t cb = (int64_t)blockIdx.z * B;

    // staging: a thread is tied to up to kDirectPos positions of each plane
    int igo[kDirectPos], ilo[kDirectPos], dgo[kDirectPos], dlo[kDirectPos];
#pragma unroll
    for (int i = 0; i < kDirectPos; ++i) {
        const int e = tid + 256 * i;
        const int yi = e / g.iw, xi = e - yi * g.iw;
        igo[i] = e < ihw ? e : -1;
        ilo[i] = (yi + g.pad) * IWP + xi + g.pad;
        const int yo = e / g.ow, xo = e - yo * g.ow;
        dgo[i] = e < ohw ? e : -1;
        dlo[i] = yo * OWS + xo;
    }
    for (int e = tid; e < SPW * iplane; e += 256) Ism[e] = 0.f;

    float acc[KS], dsum = 0.f;
#pragma unroll
    for (int k = 0; k < KS; ++k) acc[k] = 0.f;

    // the planes of the next samples are fetched into registers before the products of the
    // current ones start and go to LDS after them
    float vi[kDirectSlots][kDirectPos], vd[kDirectSlots][kDirectPos];
    auto fetch = [&](int b0) {
#pragma unroll
        for (int sl = 0; sl < kDirectSlots; ++sl) {
            if (sl < SPW) {
                const int b = b0 + sl < B ? b0 + sl : 0;
                const float *ib = in + (cb + b) * g.in_size + (int64_t)ic * ihw;
                const float *db = dout + (cb + b) * g.out_size + (int64_t)oc * ohw;
#pragma unroll
                for (int i = 0; i < kDirectPos; ++i) {
                    vi[sl][i] = ib[igo[i] >= 0 ? igo[i] : 0];
                    vd[sl][i] = db[dgo[i] >= 0 ? dgo[i] : 0];
                }
            }
        }
    };
    constexpr int CH = 2 * KS;   // pixels per step of the row walk (a multiple of KS: the window's
                                 // registers keep their places)
    fetch(0);
    for (int b0 = 0; b0 < B; b0 += SPW) {
        __syncthreads();   // the products of the previous samples are done (first pass: borders are zero)
#pragma unroll
        for (int sl = 0; sl < kDirectSlots; ++sl) {
            if (sl < SPW) {
                const bool bok = b0 + sl < B;
#pragma unroll
                for (int i = 0; i < kDirectPos; ++i) {
                    if (igo[i] >= 0) Ism[sl * iplane + ilo[i]] = bok ? vi[sl][i] : 0.f;
                    if (dgo[i] >= 0) Dsm[sl * dplane + dlo[i]] = bok ? vd[sl][i] : 0.f;
                }
            }
        }
        __syncthreads();
        if (b0 + SPW < B) fetch(b0 + SPW);
        if (active) {
            const float *Irow = Ism + slot * iplane + (y + ky) * IWP;
            const float *Drow = Dsm + slot * dplane + y * OWS;
            float w[KS];
#pragma unroll
            for (int j = 0; j < KS - 1; ++j) w[j] = Irow[j];
            for (int x0 = 0; x0 < g.ow; x0 += CH) {
                float dv[CH], nv[CH];
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    const int x = x0 + j < g.ow ? x0 + j : g.ow - 1;   // beyond the row: d = 0
                    nv[j] = Irow[x + KS - 1];
                    dv[j] = Drow[x];
                    if (x0 + j >= g.ow) dv[j] = 0.f;
                }
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    w[(j + KS - 1) % KS] = nv[j];
                    dsum += dv[j];
#pragma unroll
                    for (int kx = 0; kx < KS; ++kx) acc[kx] += dv[j] * w[(j + kx) % KS];
                }
            }
        }
    }
    if (active) {
#pragma unroll
        for (int kx = 0; kx < KS; ++kx) red[tid * (KS + 1) + kx] = acc[kx];
        red[tid * (KS + 1) + KS] = dsum;
    }
    __syncthreads();
    const float invB = 1.0f / (float)B;
    if (tid < KS * KS) {
        const int fy = tid / KS, fx = tid - fy * KS;
        float sum = 0.f;
        for (int sl = 0; sl < SPW; ++sl)
            for (int yy = 0; yy < g.oh; ++yy) sum += red[(sl * rows + fy * g.oh + yy) * (KS + 1) + fx];
        sum *= invB;
        const int64_t wi = g.w_off + ((int64_t)(oc * g.ic + ic) * KS + fy) * KS + fx;
        p.W[wi] -= p.eta * sum;
        p.U[wi] += sum;
    } else if (tid == KS * KS && ic == 0) {
        float sum = 0.f;
        for (int sl = 0; sl < SPW; ++sl)
            for (int yy = 0; yy < g.oh; ++yy) sum += red[(sl * rows + yy) * (KS + 1) + KS];
        sum *= invB;
        p.W[g.b_off + oc] -= p.eta * sum;
        p.U[g.b_off + oc] += sum;
    }
}

static size_t conv_wgrad_direct_lds(const LayerGeom &g) {
    const int IWP = (g.iw + 2 * g.pad) | 1, IHP = g.ih + 2 * g.pad, OWS = g.ow | 1;
    const int rows = g.k * g.oh;
    if (rows > 256) return 0;
    const int SPW = 256 / rows < kDirectSlots ? 256 / rows : kDirectSlots;
    return sizeof(float) * ((size_t)SPW * (IHP * IWP + g.oh * OWS) + (size_t)SPW * rows * (g.k + 1));
}

// few channels (the matrix tiles of the MFMA kernel would be mostly padding), small planes
static bool conv_wgrad_direct_ok(const LayerGeom &g) {
    if (!(g.k == 3 || g.k == 5)) return false;
    if (g.ic * g.k * g.k + 1 > 32 || g.oc > 16) return false;
    if (g.ih * g.iw > 256 * kDirectPos || g.oh * g.ow > 256 * kDirectPos) return false;
    if (g.ow != g.iw + 2 * g.pad - g.k + 1 || g.oh != g.ih + 2 * g.pad - g.k + 1) return false;
    const size_t lds = conv_wgrad_direct_lds(g);
    return lds > 0 && lds <= 64 * 1024;
}

static hipError_t launch_conv_wgrad_direct(hipStream_t s, Profiler *prof, const RoundParams *dp, int nact,
                                           int u, int B, const LayerGeom &g, const float *in,
                                           const float *dout) {
    dim3 grid((unsigned)g.oc, (unsigned)g.ic, (unsigned)nact);
    const size_t lds = conv_wgrad_direct_lds(g);
    if (g.k == 3)
        AET_TIMED(F_CONV_BWD_WEIGHT, k_conv_wgrad_direct<3><<<grid, 256, lds, s>>>(dp, u, B, g, in, dout));
    else
        AET_TIMED(F_CONV_BWD_WEIGHT, k_conv_wgrad_direct<5><<<grid, 256, lds, s>>>(dp, u, B, g, in, dout));
    return hipGetLastError();
}

static hipError_t conv_dispatch(int ks, hipStream_t s, Profiler *prof, const RoundParams *dp, int nact, int u,
                                int B, const LayerGeom &g, int which, const float *a,
                                const float *b, float *c, const float *mask, bool mfma) {
    if (which < 2 && mfma && conv_mfma_supported(g, which == 1))
        return launch_conv_mfma(s, prof, dp, nact, u, B, g, which == 1, a, c, mask);
    if (which == 2 && mfma && conv_wgrad_direct_ok(g))
        return launch_conv_wgrad_direct(s, prof, dp, nact, u, B, g, a, b);
    if (which == 2 && mfma && c && conv_wgrad_mfma_supported(g, B))
        return launch_conv_wgrad_mfma(s, prof, dp, nact, u, B, g, a, b, c);
    switch (ks) {
        case 1: return conv_step<1>(s, prof, dp, nact, u, B, g, which, a, b, c, mask);
        case 2: return conv_step<2>(s, prof, dp, nact, u, B, g, which, a, b, c, mask);
        case 3: return conv_step<3>(s, prof, dp, nact, u, B, g, which, a, b, c, mask);
        case 5: return conv_step<5>(s, prof, dp, nact, u, B, g, which, a, b, c, mask);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_layer_step(hipStream_t s, Profiler *prof, const RoundParams *dp, int nact, int u,
                             const LayerGeom *lay, int L, int B, const LayerScratch &sc) {
    if (nact <= 0) return hipSuccess;
    {
        const int D = (int)lay[0].in_size;
        dim3 grid((D + 255) / 256, B, nact);
        AET_TIMED(F_GATHER, k_gather<<<grid, 256, 0, s>>>(dp, u, B, D, sc.act[0], sc.labels));
        AET_RETURN_IF(hipGetLastError());
    }
    for (int l = 0; l < L; ++l) {
        const LayerGeom &g = lay[l];
        if (g.type == 0) {
            AET_RETURN_IF(conv_dispatch(g.k, s, prof, dp, nact, u, B, g, 0, sc.act[l], nullptr,
                                        sc.act[l + 1], nullptr, !sc.plain));
        } else if (g.type == 1) {
            if (pool_pairs(g)) {
                dim3 grid((unsigned)((g.out_size / 2 + 255) / 256), B, nact);
                AET_TIMED(F_POOL_FWD, k_pool_fwd_pair<<<grid, 256, 0, s>>>(dp, u, B, g, sc.act[l], sc.act[l + 1], sc.amax[l]));
            } else {
                dim3 grid((unsigned)((g.out_size + 255) / 256), B, nact);
                AET_TIMED(F_POOL_FWD, k_pool_fwd<<<grid, 256, 0, s>>>(dp, u, B, g, sc.act[l], sc.act[l + 1], sc.amax[l]));
            }
            AET_RETURN_IF(hipGetLastError());
        } else if (!sc.plain) {
            AET_RETURN_IF(launch_dense_mfma(s, prof, 0, dp, nact, u, B, (int)g.in_size, g.oc, g.w_off, g.b_off,
                                            g.relu, sc.act[l], nullptr, sc.act[l + 1], nullptr));
        } else {
            dim3 grid((g.oc + 3) / 4, 1, nact);
            AET_TIMED(F_DENSE_FWD, k_dense_fwd<<<grid, 256, 0, s>>>(dp, u, B, (int)g.in_size, g.oc, g.w_off, g.b_off,
                                                                    g.relu, sc.act[l], sc.act[l + 1]));
            AET_RETURN_IF(hipGetLastError());
        }
    }
    AET_TIMED(F_SOFTMAX_CE, k_softmax_ce<<<nact, 256, 0, s>>>(dp, u, B, lay[L - 1].oc, sc.act[L], sc.labels, sc.del[L]));
    AET_RETURN_IF(hipGetLastError());
    for (int l = L - 1; l >= 0; --l) {
        const LayerGeom &g = lay[l];
        // the gradient handed to act[l] is masked by the ReLU of the layer that produced it
        const float *mask = (l > 0 && lay[l - 1].relu) ? sc.act[l] : nullptr;
        if (g.type == 0) {
            if (l > 0)
                AET_RETURN_IF(conv_dispatch(g.k, s, prof, dp, nact, u, B, g, 1, sc.del[l + 1], nullptr,
                                            sc.del[l], mask, !sc.plain));
            AET_RETURN_IF(conv_dispatch(g.k, s, prof, dp, nact, u, B, g, 2, sc.act[l], sc.del[l + 1],
                                        sc.wgrad, nullptr, !sc.plain));
        } else if (g.type == 1) {
            if (l > 0) {
                if (pool_pairs(g)) {
                    dim3 grid((unsigned)((g.out_size / 2 + 255) / 256), B, nact);
                    AET_TIMED(F_POOL_BWD, k_pool_bwd_pair<<<grid, 256, 0, s>>>(dp, u, B, g, sc.del[l + 1], sc.amax[l], sc.del[l], mask));
                } else {
                    dim3 grid((unsigned)((g.out_size + 255) / 256), B, nact);
                    AET_TIMED(F_POOL_BWD, k_pool_bwd<<<grid, 256, 0, s>>>(dp, u, B, g, sc.del[l + 1], sc.amax[l], sc.del[l], mask));
                }
                AET_RETURN_IF(hipGetLastError());
            }
        } else if (!sc.plain) {
            const int K = (int)g.in_size;
            if (l > 0)
                AET_RETURN_IF(launch_dense_mfma(s, prof, 1, dp, nact, u, B, K, g.oc, g.w_off, g.b_off, 0,
                                                sc.del[l + 1], nullptr, sc.del[l], mask));
            AET_RETURN_IF(launch_dense_mfma(s, prof, 2, dp, nact, u, B, K, g.oc, g.w_off, g.b_off, 0,
                                            sc.act[l], sc.del[l + 1], nullptr, nullptr));
        } else {
            const int K = (int)g.in_size;
            if (l > 0) {
                dim3 grid((K + 255) / 256, B, nact);
                AET_TIMED(F_DENSE_BWD_DATA, k_dense_bwd_data<<<grid, 256, 0, s>>>(dp, u, B, K, g.oc, g.w_off, sc.del[l + 1], sc.del[l], mask));
                AET_RETURN_IF(hipGetLastError());
            }
            dim3 grid((K + 255) / 256, g.oc, nact);
            AET_TIMED(F_DENSE_BWD_WEIGHT, k_dense_bwd_weight<<<grid, 256, 0, s>>>(dp, u, B, K, g.oc, g.w_off, g.b_off, sc.act[l], sc.del[l + 1]));
            AET_RETURN_IF(hipGetLastError());
        }
    }
    return hipSuccess;
}

__global__ void k_debug_indices(uint64_t key, int64_t q0, int count, uint32_t n_samples,
                                int32_t *__restrict__ dst) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) dst[i] = (int32_t)sample_row(key, (uint64_t)(q0 + i), n_samples);
}

hipError_t launch_debug_indices(hipStream_t s, uint64_t key, int64_t q0, int count,
                                uint32_t n_samples, int32_t *dst) {
    if (count <= 0) return hipSuccess;
    k_debug_indices<<<(count + 255) / 256, 256, 0, s>>>(key, q0, count, n_samples, dst);
    return hipGetLastError();
}

}  // namespace aet
