// Convolution layers of the layer-by-layer engine on the matrix cores (fp32 MFMA 16x16x4),
// as implicit GEMMs over tiles staged in LDS.  Stride 1, square kernels, zero padding.
//
// Forward and backward-data are the same kernel:
//   dst[dc][y][x] = sum_{sc,ky,kx} src[sc][y+ky-P][x+kx-P] * Wt[dc][sc][ky][kx]
//   forward:        src = layer input,  dst = layer output, P = pad,
//                   Wt[dc][sc][ky][kx] = W[dc][sc][ky][kx], then bias and ReLU;
//   backward-data:  src = d(output),    dst = d(input),     P = K-1-pad,
//                   Wt[dc][sc][ky][kx] = W[sc][dc][K-1-ky][K-1-kx], then the ReLU mask of the
//                   layer below.
// GEMM view: M = pixels (tiles of 16 consecutive x), N = dst channels (tiles of 16),
// K = (sc, ky, kx), walked in chunks of 8 source channels.  A workgroup owns R dst rows of
// one sample (8 M tiles), all dst channels of its N block; each of its 4 waves owns 2 M
// tiles and all N tiles.
//
// Backward-weight (g = sum over the mini-batch and all pixels of d(output) x input patch):
//   M = output channels, N = (ci, ky, kx) plus one extra column for the bias, K = pixels.
//   A workgroup accumulates its share of (sample, row block) work items in registers and
//   writes one partial result; a second kernel adds the partials in fixed order, scales by
//   1/B and applies  w <- w - eta g,  U <- U + g  (the gradient itself is never stored
//   in the canonical layout).
#include <type_traits>

#include "aet_device.h"
#include "aet_internal.h"

namespace aet {

typedef float f4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f4 mfma16x16x4(float a, float b, f4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// dword 3 of a raw buffer descriptor for 32-bit untyped accesses on this part
constexpr int kBufferFlags = 0x00020000;
constexpr uint32_t kNowhere = 0x80000000u;   // a byte offset no buffer here reaches: reads as zero

constexpr int kCch = 8;    // source channels per K chunk, at most (layers with fewer use 1, 2 or 4)

struct ConvDir {
    int SC, DC;          // source / destination channels
    int SH, SW, DH, DW;  // source / destination height and width
    int P;               // padding in this direction
    int R;               // dst rows per workgroup
    int MPR;             // M tiles (16 columns) per dst row
    int NT;              // N tiles (16 dst channels) per workgroup
    int CCH;             // source channels per K chunk: 1, 2, 4 or 8
    int rowsT, SWP;      // rows and padded width of the staged source tile
    int PL;              // floats between the tile's channel planes in LDS (16 mod 32)
    int npos;            // tile positions one thread stages: 1, 2 or 3
    int vec;             // rows and weight runs are 16-byte aligned: the four-pixel staging
    int nslot, sgrp;     // ... its groups of four pixels per channel plane; channel groups of threads
    int64_t src_size, dst_size;  // floats per sample
    int64_t w_off, b_off;
    int ic, oc;          // the layer's own channel counts (weight layout W[oc][ic][K][K])
    int relu;
};

// CCH: source channels per K chunk (1, 2, 4 or 8: the smallest that holds the layer's source
// channels, so that a 1- or 3-channel input does not multiply seven or five channels of zeros).
// NT: N tiles (16 destination channels each) per workgroup: 1, 2 or 4.
// NPOS: positions of the source tile one thread stages, at most: 1 (tiles of up to 256
// positions, the common case: no loop, no spare registers) or 3.
//
// Order of the chunk's K elements.  CCH >= 4: k = ((cq*KS + ky)*KS + kx)*4 + c4, channel
// 4*cq + c4: the four K elements of one matrix instruction are four channels at one filter
// tap, so a lane's source address is its base plus a number that is the same for the whole
// wave.  CCH < 4: k = c*KS*KS + ky*KS + kx, each lane keeps the tile offsets of its K
// elements in registers.  In both cases the operands of the next step are read from LDS
// before the products of the current step are issued.
//
// VEC (chunks of 8 channels, source rows and weight runs 16-byte aligned, no partial chunk):
// staging moves 16 bytes per load.  A thread is tied to four consecutive pixels of one tile
// row and walks channels; for the weights to four consecutive elements of the memory run and
// walks destination channels (forward) or source channels (backward-data).  The tile's halo
// columns never change and are zeroed once.
template <int KS, bool BWD, int CCH, int NT, int NPOS, bool VEC>
__global__ void __launch_bounds__(256, VEC ? 4 : 1)   // VEC: at most 128 registers, 4 workgroups per CU
k_conv_mfma(const RoundParams *__restrict__ rp, int u, int B, ConvDir g, const float *__restrict__ src,
            float *__restrict__ dst, const float *__restrict__ mask_src) {
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    constexpr int KSQ = KS * KS;
    constexpr int KCHR = CCH * KSQ;          // K elements per chunk
    constexpr int KCH = (KCHR + 3) / 4 * 4;  // ... rounded up to whole contraction steps (zero weights)
    constexpr int KCHP = KCH + 2;            // weight row in LDS: KCHP / 2 odd, no bank conflicts among 16 rows
    constexpr int STEPS = KCH / 4;
    constexpr bool CF = CCH >= 4;            // channels fastest
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 15, lg = lane >> 4;
    const int nblocks = (g.DC + 16 * NT - 1) / (16 * NT);
    const int nblk = blockIdx.x % nblocks, rblk = blockIdx.x / nblocks;
    const int y0 = rblk * g.R;
    const int dc0 = nblk * 16 * NT;
    const int64_t sample = (int64_t)blockIdx.z * B + blockIdx.y;
    // range-checked buffers: the sample's source planes and the layer's weights; an offset
    // beyond them (kNowhere, or a channel beyond the last) reads zero without touching memory
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(src) + sample * g.src_size, 0, (int)(4 * g.src_size), kBufferFlags);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        p.W + g.w_off, 0, 4 * g.ic * g.oc * KS * KS, kBufferFlags);
    auto bload = [](__amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
        return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)byte_off, 0, 0));
    };
    auto bload4 = [](__amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
        return __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, 0));
    };

    extern __shared__ float smem[];
    const int tile_plane = g.rowsT * g.SWP;
    const int PL = g.PL;                        // plane stride: 16 mod 32, so that the four lane
    float *Ssm = smem;                          // groups of an A operand fall into distinct banks
    float *Wsm = Ssm + CCH * PL;                // [16*NT][KCHP]

    // the wave's two M tiles: (row, column chunk) inside the workgroup's block
    int abase[2];
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const int mt = 2 * wave + m;
        const int row = mt / g.MPR, cch = mt - row * g.MPR;
        abase[m] = row * g.SWP + 16 * cch + li + (CF ? lg * PL : 0);
    }
    int ko[CF ? 1 : STEPS];
    if (!CF) {
#pragma unroll
        for (int st = 0; st < STEPS; ++st) {
            const int k = 4 * st + lg;
            const int c = k / KSQ, r = k - c * KSQ;
            ko[CF ? 0 : st] = k < KCHR ? c * PL + (r / KS) * g.SWP + (r % KS) : 0;  // padding: weight 0
        }
    }
    const int bbase = li * KCHP + lg;
    f4 acc[2][NT];
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n) acc[m][n] = f4{0.f, 0.f, 0.f, 0.f};

    // Staging without per-element index arithmetic and without branches: a thread is tied to
    // up to 3 positions of the source tile and walks the chunk's channels, and to one K
    // element of the weight chunk and walks the destination channels; what lies outside asks
    // the range-checked buffers for an offset beyond their end and comes back as zero.
    const uint32_t shw = 4u * (uint32_t)(g.SH * g.SW);   // bytes per source channel
    uint32_t soff[NPOS];
    bool sok[NPOS];
#pragma unroll
    for (int i = 0; i < NPOS; ++i) {
        const int pos = tid + 256 * i;
        const int ty = pos / g.SWP, tx = pos - ty * g.SWP;
        const int sy = y0 + ty - g.P, sx = tx - g.P;
        sok[i] = pos < tile_plane && (unsigned)sy < (unsigned)g.SH && (unsigned)sx < (unsigned)g.SW;
        soff[i] = sok[i] ? 4u * (uint32_t)(sy * g.SW + sx) : kNowhere;   // byte offset in the sample
    }
    // Weights of a chunk, Wsm[d][k].  Threads follow the memory order, so that a wave's loads
    // are consecutive addresses, and scatter into the K order of the chunk in LDS.
    //   forward, Wt = W[dc][sc][ky][kx]: for one dc the chunk is a run of CCH*KS*KS floats;
    //     a thread is tied to one element of the run and walks the destination channels.
    //   backward-data, Wt[dc][sc][ky][kx] = W[sc][dc][K-1-ky][K-1-kx]: for one sc the
    //     workgroup's destination channels are a run of 16*NT*KS*KS floats; a thread is tied
    //     to up to NPB elements of the run and walks the chunk's source channels.
    constexpr int nd = 16 * NT;
    const int dlim = min(nd, g.DC - dc0);                // destination channels that exist
    auto kcol = [](int c, int tap) { return CF ? ((c >> 2) * KSQ + tap) * 4 + (c & 3) : c * KSQ + tap; };
    constexpr int WG_ = 256 / KCH > 0 ? 256 / KCH : 1;   // forward: dst-channel groups
    const int wm = tid % KCH, wd0 = tid / KCH;           // forward: element of the run, first dst channel
    const int wc = wm / KSQ, wr = wm - wc * KSQ;
    const bool wactive = wd0 < WG_;
    const bool wreal = wm < KCHR;                        // not one of the padding columns
    const int wcol = wreal ? kcol(wc, wr) : wm;
    const uint32_t wdstep = (uint32_t)(g.ic * KSQ);
    const uint32_t wbase = (uint32_t)(dc0 * g.ic * KSQ + wm);
    constexpr int NPB = (nd * KSQ + 255) / 256;          // backward-data: elements of the run per thread
    uint32_t boff[BWD ? NPB : 1];
    int blds[BWD ? NPB : 1];
    if (BWD) {
#pragma unroll
        for (int i = 0; i < NPB; ++i) {
            const int j = tid + 256 * i;
            const int d = j / KSQ, tm = j - d * KSQ;
            const bool ok = j < nd * KSQ && d < dlim;
            boff[BWD ? i : 0] = ok ? (uint32_t)(dc0 * KSQ + j) : 0xffffffffu;
            blds[BWD ? i : 0] = j < nd * KSQ ? d * KCHP + kcol(0, KSQ - 1 - tm) : -1;
        }
        if constexpr (KCH > KCHR)   // padding columns: zero weights, written once
            for (int e = tid; e < nd * (KCH - KCHR); e += 256)
                Wsm[(e / (KCH - KCHR)) * KCHP + KCHR + e % (KCH - KCHR)] = 0.f;
    }
    const uint32_t bcstep = (uint32_t)(g.ic * KSQ);

    // The four-pixel staging.  Source tile: thread = (group of four pixels, channel group),
    // channels vcg, vcg + sgrp.  Forward weights: thread = (four elements fq of the run of one
    // destination channel, first destination channel fd0).  Backward-data weights: thread =
    // (four elements gq of the run of one source channel, channel group gcg).
    constexpr int kTurnsS = 2;
    constexpr int QF = KCHR / 4, WGF = 256 / (QF > 0 ? QF : 1), NWF = (nd + WGF - 1) / WGF;
    constexpr int QB = nd * KSQ / 4;
    constexpr int NGB = 256 / QB < 1 ? 1 : (256 / QB > CCH ? CCH : 256 / QB);
    constexpr int NBT = (CCH + NGB - 1) / NGB;
    uint32_t voff[kTurnsS];
    bool vst[kTurnsS];
    int vlds = 0, vstep = 0, fcol[4], gl[4];
    int fq = 0, fd0 = 0, gq = 0, gcg = 0;
    if constexpr (VEC) {
        const int sw4 = g.SW >> 2;
        const int vslot = tid % g.nslot, vcg = tid / g.nslot;
        const int vty = vslot / sw4, vxq = vslot - vty * sw4;
        const int vsy = y0 + vty - g.P;
#pragma unroll
        for (int j = 0; j < kTurnsS; ++j) {
            const int c = vcg + g.sgrp * j;
            vst[j] = vcg < g.sgrp && c < CCH;
            voff[j] = (vst[j] && (unsigned)vsy < (unsigned)g.SH)
                          ? 4u * (uint32_t)(vsy * g.SW + 4 * vxq) + (uint32_t)c * shw : kNowhere;
        }
        vlds = vcg * PL + vty * g.SWP + g.P + 4 * vxq;
        vstep = g.sgrp * PL;
        fq = tid % QF; fd0 = tid / QF;
        gq = tid % QB; gcg = tid / QB;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int m = 4 * fq + e;
            fcol[e] = kcol(m / KSQ, m % KSQ);
            const int j = 4 * gq + e;
            gl[e] = (j / KSQ) * KCHP + kcol(0, KSQ - 1 - j % KSQ);
        }
        // halo columns: P on the left, the rest on the right of the image's columns
        const int hw = g.SWP - g.SW, per = g.rowsT * hw;
        for (int e = tid; e < CCH * per; e += 256) {
            const int c = e / per, r = e - c * per;
            const int ty = r / hw, h = r - ty * hw;
            Ssm[c * PL + ty * g.SWP + (h < g.P ? h : g.SW + h)] = 0.f;
        }
    }
    const uint32_t fbase = (uint32_t)(dc0 * g.ic * KSQ + 4 * fq);
    const uint32_t gbase = (uint32_t)(dc0 * KSQ + 4 * gq);

    // All loads of a chunk (source tile and weights) are issued before the first of them is
    // stored to LDS: one memory round trip per chunk.
    constexpr int NWL = (nd + WG_ - 1) / WG_;            // forward: destination channels per thread
    constexpr int NWV = BWD ? NPB * CCH : NWL;
    for (int c0 = 0; c0 < g.SC; c0 += CCH) {
        __syncthreads();   // the products of the previous chunk are done with the tiles
        if constexpr (VEC) {
            f4 sv4[kTurnsS], wv4[BWD ? NBT : NWF];
#pragma unroll
            for (int j = 0; j < kTurnsS; ++j) sv4[j] = bload4(rs, voff[j] + (uint32_t)c0 * shw);
            if (BWD) {
#pragma unroll
                for (int j = 0; j < NBT; ++j) {
                    const int c = gcg + NGB * j;
                    const bool ok = gcg < NGB && c < CCH;
                    wv4[j] = bload4(rw, ok ? 4u * (gbase + (uint32_t)(c0 + c) * bcstep) : kNowhere);
                }
            } else {
                const int lim = fd0 < WGF ? dlim : 0;
                const uint32_t q = fbase + (uint32_t)c0 * KSQ;
#pragma unroll
                for (int j = 0; j < NWF; ++j) {
                    const int d = fd0 + WGF * j;
                    wv4[j] = bload4(rw, d < lim ? 4u * (q + (uint32_t)d * wdstep) : kNowhere);
                }
            }
#pragma unroll
            for (int j = 0; j < kTurnsS; ++j)
                if (vst[j]) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) Ssm[vlds + j * vstep + e] = sv4[j][e];
                }
            if (BWD) {
#pragma unroll
                for (int j = 0; j < NBT; ++j) {
                    const int c = gcg + NGB * j;
                    if (gcg < NGB && c < CCH) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) Wsm[gl[e] + kcol(c, 0)] = wv4[j][e];
                    }
                }
            } else if (fd0 < WGF) {
#pragma unroll
                for (int j = 0; j < NWF; ++j) {
                    const int d = fd0 + WGF * j;
                    if (d < nd) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) Wsm[d * KCHP + fcol[e]] = wv4[j][e];
                    }
                }
            }
        } else {
        float sv[NPOS][CCH], wv[NWV];
#pragma unroll
        for (int i = 0; i < NPOS; ++i)
            if (i < g.npos) {
#pragma unroll
                for (int c = 0; c < CCH; ++c)
                    sv[i][c] = bload(rs, soff[i] + (uint32_t)(c0 + c) * shw);   // channels beyond SC lie beyond the sample
            }
        if (BWD) {
#pragma unroll
            for (int i = 0; i < NPB; ++i)
#pragma unroll
                for (int c = 0; c < CCH; ++c) {
                    const bool ok = boff[BWD ? i : 0] != 0xffffffffu && c0 + c < g.SC;
                    wv[BWD ? i * CCH + c : 0] = bload(rw, ok ? 4u * (boff[BWD ? i : 0] + (uint32_t)(c0 + c) * bcstep) : kNowhere);
                }
        } else {
            const int lim = (wactive && wreal && c0 + wc < g.SC) ? dlim : 0;
            const uint32_t q = wbase + (uint32_t)c0 * KSQ;
#pragma unroll
            for (int j = 0; j < NWL; ++j) {
                const int d = wd0 + WG_ * j;
                wv[BWD ? 0 : j] = bload(rw, d < lim ? 4u * (q + (uint32_t)d * wdstep) : kNowhere);
            }
        }
#pragma unroll
        for (int i = 0; i < NPOS; ++i)
            if (i < g.npos && tid + 256 * i < tile_plane) {
#pragma unroll
                for (int c = 0; c < CCH; ++c)
                    Ssm[c * PL + tid + 256 * i] = sv[i][c];
            }
        if (BWD) {
#pragma unroll
            for (int i = 0; i < NPB; ++i)
                if (blds[BWD ? i : 0] >= 0) {
#pragma unroll
                    for (int c = 0; c < CCH; ++c) Wsm[blds[BWD ? i : 0] + kcol(c, 0)] = wv[BWD ? i * CCH + c : 0];
                }
        } else if (wactive) {
#pragma unroll
            for (int j = 0; j < NWL; ++j) {
                const int d = wd0 + WG_ * j;
                if (d < nd) Wsm[d * KCHP + wcol] = wv[BWD ? 0 : j];
            }
        }
        }
        __syncthreads();
        float a[2][2], bv[2][NT];
        auto operands = [&](int st, int set) {
            int off;
            if (CF) {
                const int t = st / KS;
                off = (t / KS) * 4 * PL + (t % KS) * g.SWP + st % KS;
            } else {
                off = ko[CF ? 0 : st];
            }
            a[set][0] = Ssm[abase[0] + off];
            a[set][1] = Ssm[abase[1] + off];
#pragma unroll
            for (int n = 0; n < NT; ++n) bv[set][n] = Wsm[bbase + 16 * n * KCHP + 4 * st];
        };
        operands(0, 0);
#pragma unroll
        for (int st = 0; st < STEPS; ++st) {
            if (st + 1 < STEPS) operands(st + 1, (st + 1) & 1);
#pragma unroll
            for (int n = 0; n < NT; ++n) {
                acc[0][n] = mfma16x16x4(a[st & 1][0], bv[st & 1][n], acc[0][n]);
                acc[1][n] = mfma16x16x4(a[st & 1][1], bv[st & 1][n], acc[1][n]);
            }
        }
    }

    // epilogue: lane holds dst channel dc0+16n+li, 4 consecutive x
    const gf_ptr dg = as_global(dst) + sample * g.dst_size;
    const gcf_ptr mg = mask_src ? as_global(mask_src) + sample * g.dst_size : nullptr;
    const bool vec = (g.DW & 3) == 0;   // whole groups of 4 pixels, 16-byte aligned
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const int mt = 2 * wave + m;
        const int row = mt / g.MPR, cch = mt - row * g.MPR;
        const int y = y0 + row;
        if (row >= g.R || y >= g.DH) continue;
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            const int dc = dc0 + 16 * n + li;
            if (dc >= g.DC) continue;
            const float bias = BWD ? 0.f : as_global(p.W)[g.b_off + dc];
            const int x0 = 16 * cch + 4 * lg;
            const int64_t i0 = ((int64_t)dc * g.DH + y) * g.DW + x0;
            if (vec) {
                if (x0 >= g.DW) continue;
                f4 v = acc[m][n] + bias;
                if (BWD) {
                    if (mg) {
                        const f4 k = *reinterpret_cast<const f4 __attribute__((address_space(1))) *>(mg + i0);
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (!(k[r] > 0.f)) v[r] = 0.f;
                    }
                } else if (g.relu) {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (!(v[r] > 0.f)) v[r] = 0.f;
                }
                *reinterpret_cast<f4 __attribute__((address_space(1))) *>(dg + i0) = v;
                continue;
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (x0 + r >= g.DW) continue;
                float v = acc[m][n][r] + bias;
                if (BWD) {
                    if (mg && !(mg[i0 + r] > 0.f)) v = 0.f;
                } else if (g.relu && !(v > 0.f)) {
                    v = 0.f;
                }
                dg[i0 + r] = v;
            }
        }
    }
}

static int device_cus() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
            cus = 256;
    }
    return cus;
}

static bool conv_dir(const LayerGeom &L, bool bwd, ConvDir *d, int nt_max = 4) {
    const int KS = L.k;
    if (!(KS == 3 || KS == 5)) return false;
    d->ic = L.ic; d->oc = L.oc; d->relu = L.relu;
    d->w_off = L.w_off; d->b_off = L.b_off;
    if (!bwd) {
        d->SC = L.ic; d->DC = L.oc; d->SH = L.ih; d->SW = L.iw; d->DH = L.oh; d->DW = L.ow; d->P = L.pad;
        d->src_size = L.in_size; d->dst_size = L.out_size;
    } else {
        d->SC = L.oc; d->DC = L.ic; d->SH = L.oh; d->SW = L.ow; d->DH = L.ih; d->DW = L.iw; d->P = KS - 1 - L.pad;
        d->src_size = L.out_size; d->dst_size = L.in_size;
    }
    if (d->DW > 128) return false;
    d->MPR = (d->DW + 15) / 16;
    if (d->MPR > 8) return false;
    d->R = 8 / d->MPR;
    if (d->R < 1) d->R = 1;
    // the 4 waves own 8 M tiles; with MPR in {3, 5, 6, 7} some tiles stay unused
    d->NT = (d->DC + 15) / 16;
    d->NT = d->NT <= 1 ? 1 : d->NT <= 2 ? 2 : 4;
    if (d->NT > nt_max) d->NT = nt_max;
    d->CCH = d->SC <= 1 ? 1 : d->SC <= 2 ? 2 : d->SC <= 4 ? 4 : kCch;
    d->rowsT = d->R + KS - 1;
    d->SWP = 16 * d->MPR + KS - 1;
    d->SWP += (d->SWP & 1) ? 0 : 1;  // odd row stride: fewer LDS bank conflicts
    const int tile_plane = d->rowsT * d->SWP;
    d->PL = tile_plane + ((16 - tile_plane % 32 + 32) % 32);
    d->npos = (tile_plane + 255) / 256;
    if (d->npos > 3) return false;
    if (d->src_size >= (int64_t)1 << 28 || (int64_t)L.oc * L.ic * KS * KS >= (int64_t)1 << 28) return false;   // 32-bit byte offsets
    // the four-pixel staging: whole chunks of 8 channels, rows and weight runs 16-byte aligned,
    // whole blocks of destination channels, at most 64 groups of four pixels per plane (two
    // turns of at least 4 channel groups of threads cover the chunk's 8 channels)
    d->nslot = d->rowsT * (d->SW >> 2);
    d->sgrp = d->nslot > 0 ? 256 / d->nslot : 0;
    if (d->sgrp > kCch) d->sgrp = kCch;
    d->vec = KS == 3 && d->CCH == kCch && d->SC % kCch == 0 && (d->SW & 3) == 0 && d->sgrp >= 4 &&
             (L.ic & 3) == 0 && (L.w_off & 3) == 0 && d->DC % (16 * d->NT) == 0;
    return true;
}

static size_t conv_lds_bytes(const ConvDir &d, int KS) {
    const int KCH = (d.CCH * KS * KS + 3) / 4 * 4;
    return sizeof(float) * ((size_t)d.CCH * d.PL + (size_t)16 * d.NT * (KCH + 2));
}

bool conv_mfma_supported(const LayerGeom &L, bool bwd) {
    ConvDir d;
    if (!conv_dir(L, bwd, &d)) return false;
    return conv_lds_bytes(d, L.k) <= 64 * 1024;
}

hipError_t launch_conv_mfma(hipStream_t s, Profiler *prof, const RoundParams *dp, int nact, int u, int B,
                            const LayerGeom &L, bool bwd, const float *src, float *dst,
                            const float *mask_src) {
    ConvDir d;
    if (!conv_dir(L, bwd, &d)) return hipErrorInvalidValue;
    // A launch of the widest tiling (4 N tiles, 4 resident workgroups per compute unit) that
    // has fewer than two full rounds of workgroups ends with compute units running a last
    // workgroup alone; half as wide workgroups, twice as many, fill that tail (measured on
    // launches of 10 and 12 clients: +2.5 % on the job; 1 N tile: +0.8 %).
    if (d.NT == 4 && (int64_t)((d.DH + d.R - 1) / d.R) * ((d.DC + 63) / 64) * B * nact < (int64_t)8 * device_cus() &&
        !conv_dir(L, bwd, &d, 2))
        return hipErrorInvalidValue;
    const size_t lds = conv_lds_bytes(d, L.k);
    const int nblocks = (d.DC + 16 * d.NT - 1) / (16 * d.NT);
    const int rblocks = (d.DH + d.R - 1) / d.R;
    dim3 grid((unsigned)(nblocks * rblocks), (unsigned)B, (unsigned)nact);
    const int fam = bwd ? F_CONV_BWD_DATA : F_CONV_FWD;
    const bool timed = prof && prof->on[fam];
    if (timed) prof->before(fam, s);
#define AET_CONV(KSv, CCHv, NTv, NPv)                                                                                \
    if (L.k == KSv && d.CCH == CCHv && d.NT == NTv && np == NPv) {                                                  \
        if (bwd) k_conv_mfma<KSv, true, CCHv, NTv, NPv, false><<<grid, 256, lds, s>>>(dp, u, B, d, src, dst, mask_src);  \
        else k_conv_mfma<KSv, false, CCHv, NTv, NPv, false><<<grid, 256, lds, s>>>(dp, u, B, d, src, dst, mask_src);     \
    }
#define AET_CONV_VEC(NTv)                                                                                            \
    if (np == 0 && d.NT == NTv) {                                                                                    \
        if (bwd) k_conv_mfma<3, true, 8, NTv, 1, true><<<grid, 256, lds, s>>>(dp, u, B, d, src, dst, mask_src);    \
        else k_conv_mfma<3, false, 8, NTv, 1, true><<<grid, 256, lds, s>>>(dp, u, B, d, src, dst, mask_src);       \
    }
#define AET_CONV_NT(KSv, CCHv, NPv) AET_CONV(KSv, CCHv, 1, NPv) AET_CONV(KSv, CCHv, 2, NPv) AET_CONV(KSv, CCHv, 4, NPv)
    // tiles of up to 256 positions and at least 4 channels per chunk get the one-position kernel
    const int np = d.vec ? 0 : (d.npos == 1 && d.CCH >= 4) ? 1 : 3;
    AET_CONV_VEC(1) AET_CONV_VEC(2) AET_CONV_VEC(4)
    AET_CONV_NT(3, 1, 3) AET_CONV_NT(3, 2, 3) AET_CONV_NT(3, 4, 3) AET_CONV_NT(3, 8, 3)
    AET_CONV_NT(5, 1, 3) AET_CONV_NT(5, 2, 3) AET_CONV_NT(5, 4, 3) AET_CONV_NT(5, 8, 3)
    AET_CONV_NT(3, 4, 1) AET_CONV_NT(3, 8, 1) AET_CONV_NT(5, 4, 1) AET_CONV_NT(5, 8, 1)
#undef AET_CONV_NT
#undef AET_CONV
#undef AET_CONV_VEC
    if (timed) prof->after(fam, s);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// backward-weight
// ---------------------------------------------------------------------------------------
struct WgradGeom {
    int IC, OC, IH, IW, OH, OW, pad;
    int R;            // output rows per work item
    int rowsT, SWP;   // staged input tile: rows and padded width
    int OWP;          // output width rounded up to a multiple of 4
    int KTOT;         // IC*K*K + 1 (the extra column multiplies by one: the bias)
    int NTT, MTT;     // N tiles (of 16 k) and M tiles (of 16 output channels) in total
    int MTS;          // M tiles staged in LDS (what the waves' tiling covers, >= MTT)
    int DPL;          // floats per channel of the staged d(output) tile: R*OWP padded to 4 mod 32,
                      // so that the 16 channels x 4 pixels of an A operand fall into distinct banks
    int items_per_sample, S;
    int U;            // output rows (of all work items, in order) per slice
    int gin, gd;      // channel groups of 256 threads walking the input tile / the d(output) tile
    int nq_in_all, nq_d_all;  // the longest walks: channels per input group, rows per d(output) group
    int vec;          // rows are 16-byte aligned: the four-pixels-per-thread staging
    int gin4, gd4, nq_in4, nq_d4;   // the same four numbers for that staging
    int64_t in_size, out_size, w_off, b_off;
};

constexpr int kPreIn4 = 8;  // the same for the four-pixel staging (float4 each)
constexpr int kPreD4 = 8;
constexpr int kPreIn = 32;  // input-tile elements one thread carries from one work item to the next
constexpr int kPreD = 16;   // the same for the d(output) tile

// MT x NTW accumulator tiles per wave.  WM = 1: a wave owns M tiles 0..MT-1 and N tiles
// wave, wave+4, ...; WM = 2 (few N tiles): the waves form a 2 x 2 grid, wave w owns M tiles
// w/2, w/2+2, ... and N tiles w%2, w%2+2, ...
//
// Staging: a thread is tied to one position of the tile (row, column) and walks the channels,
// so the loop has no index arithmetic and no branches; the next work item's elements are
// fetched into registers before the products of the current one start and go to LDS after them.
template <int KS, int MT, int NTW, int WM, bool VEC>
__global__ void __launch_bounds__(256)
k_conv_wgrad_mfma(const RoundParams *__restrict__ rp, int u, int B, WgradGeom g,
                  const float *__restrict__ in, const float *__restrict__ dout,
                  float *__restrict__ partial) {
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 15, lg = lane >> 4;
    const int sl = blockIdx.x;
    const int m0 = WM == 1 ? 0 : (wave >> 1);   // first M tile of the wave, stride WM
    const int n0 = WM == 1 ? wave : (wave & 1);  // first N tile of the wave, stride NS
    constexpr int NS = 4 / WM;

    extern __shared__ float smem[];
    const int plane = g.rowsT * g.SWP;
    const int CP = VEC ? g.gin4 * g.nq_in4 : g.gin * g.nq_in_all;   // channel planes the staging threads write (>= IC)
    const int DR = VEC ? g.gd4 * g.nq_d4 : g.gd * g.nq_d_all;       // d(output) rows they write (>= 16*MTS)
    float *Ism = smem;                       // [CP + 3][rowsT][SWP]; plane CP = ones, CP+1 = zeros, CP+2 = dump
    float *Dsm = Ism + (((CP + 3) * plane + 3) & ~3);   // [DR + 1][DPL], 16-byte aligned; the last row is a dump
    const int dplane = g.R * g.OWP;

    if (VEC)   // the halo columns of the channel planes are never written again: zero them once
        for (int e = tid; e < CP * plane; e += 256) Ism[e] = 0.f;
    for (int e = tid; e < 2 * plane; e += 256) Ism[CP * plane + e] = e < plane ? 1.f : 0.f;

    // B operand: lane li of N tile nt holds column k = 16*nt + li of the GEMM
    int kb[NTW];
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
        const int k = 16 * (n0 + NS * j) + li;
        int off = (CP + 1) * plane;  // zeros
        if (k < g.IC * KS * KS) {
            const int c = k / (KS * KS), r = k - c * KS * KS;
            off = c * plane + (r / KS) * g.SWP + (r % KS);
        } else if (k == g.IC * KS * KS) {
            off = CP * plane;        // ones
        }
        kb[j] = off + lg;
    }
    // A operand: lane li of M tile mt holds output channel 16*mt + li
    int ab[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) ab[m] = (16 * (m0 + WM * m) + li) * g.DPL + lg;
    f4 acc[MT][NTW];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int j = 0; j < NTW; ++j) acc[m][j] = f4{0.f, 0.f, 0.f, 0.f};

    // This thread's position in the input tile and in the d(output) tile.  The tiles are
    // fetched with range-checked buffer loads (one descriptor per sample): a lane outside
    // the image asks for an offset beyond the sample and a turn beyond the last channel
    // lands beyond it by itself; both read zero without touching memory, so the staging code
    // has no branches and no selects.  Threads beyond the last whole channel group store to a
    // dump area.
    // VEC (image rows and d(output) rows 16-byte aligned): a thread is tied to four
    // consecutive pixels of a row, one 16-byte load and one turn per channel; the halo
    // columns of the input planes stay zero from the start.
    const int gin = VEC ? g.gin4 : g.gin;        // channel groups walking the input tile
    const int islots = VEC ? g.rowsT * (g.IW >> 2) : plane;
    const int ipos = tid % islots, igrp = tid / islots;
    const int irow = VEC ? g.IW >> 2 : g.SWP;    // positions per tile row
    const int ity = ipos / irow, itx = ipos - ity * irow;
    const bool ixok = igrp < gin && (VEC || (unsigned)(itx - g.pad) < (unsigned)g.IW);
    const int gd = VEC ? g.gd4 : g.gd;
    const int dslots = VEC ? g.R * (g.OW >> 2) : dplane;
    const int dpos = tid % dslots, dgrp = tid / dslots;
    const int drow = VEC ? g.OW >> 2 : g.OWP;
    const int dr = dpos / drow, dx = dpos - dr * drow;
    const bool dxok = dgrp < gd && (VEC || dx < g.OW);
    const uint32_t ihw = (uint32_t)(g.IH * g.IW), ohw = (uint32_t)(g.OH * g.OW);
    const uint32_t icstep = 4u * (uint32_t)gin * ihw, dcstep = 4u * (uint32_t)gd * ohw;   // bytes per turn
    const int isbase = VEC ? igrp * plane + ity * g.SWP + g.pad + 4 * itx
                           : (igrp < gin ? igrp * plane + ipos : (CP + 2) * plane + ipos);
    const int isstep = (VEC || igrp < gin) ? gin * plane : 0;
    const int dsbase = VEC ? dgrp * g.DPL + dr * g.OWP + 4 * dx
                           : (dgrp < gd ? dgrp * g.DPL + dpos : DR * g.DPL + dpos);
    const int dsstep = (VEC || dgrp < gd) ? gd * g.DPL : 0;
    const int nq_in = VEC ? g.nq_in4 : g.nq_in_all, nq_d = VEC ? g.nq_d4 : g.nq_d_all;

    // the fetched elements stay untouched in registers until they go to LDS (nothing waits
    // for a load before the products start)
    constexpr int PI = VEC ? kPreIn4 : kPreIn, PD = VEC ? kPreD4 : kPreD;
    typedef typename std::conditional<VEC, f4, float>::type stage_t;
    stage_t pin[PI], pd[PD];
    const int items = B * g.items_per_sample;
    auto bload = [](__amdgpu_buffer_rsrc_t r, uint32_t off) -> stage_t {
        if constexpr (VEC) return __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0));
        else return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, 0));
    };
    auto fetch = [&](int it) {
        const int b = it / g.items_per_sample, rb = it - b * g.items_per_sample;
        const int y0 = rb * g.R;
        const int64_t sample = (int64_t)blockIdx.z * B + b;
        const __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float *>(in) + sample * g.in_size, 0, (int)(4 * g.in_size), kBufferFlags);
        const __amdgpu_buffer_rsrc_t rd = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float *>(dout) + sample * g.out_size, 0, (int)(4 * g.out_size), kBufferFlags);
        const int sy = y0 + ity - g.pad;
        const bool iok = ixok && (unsigned)sy < (unsigned)g.IH;
        const int sx = VEC ? 4 * itx : itx - g.pad;
        const uint32_t ivo = iok ? 4u * ((uint32_t)igrp * ihw + (uint32_t)(sy * g.IW + sx)) : kNowhere;
#pragma unroll
        for (int q = 0; q < PI; ++q)
            if (q < nq_in) pin[q] = bload(rin, ivo + (uint32_t)q * icstep);
        const bool dok = dxok && y0 + dr < g.OH;
        const uint32_t dvo = dok ? 4u * ((uint32_t)dgrp * ohw + (uint32_t)((y0 + dr) * g.OW + (VEC ? 4 * dx : dx))) : kNowhere;
#pragma unroll
        for (int q = 0; q < PD; ++q)
            if (q < nq_d) pd[q] = bload(rd, dvo + (uint32_t)q * dcstep);
    };
    auto stash = [&]() {   // the fetched tiles go to LDS
        if constexpr (VEC) {
            if (igrp < gin) {
#pragma unroll
                for (int q = 0; q < PI; ++q)
                    if (q < nq_in) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) Ism[isbase + q * isstep + e] = pin[q][e];
                    }
            }
            if (dgrp < gd) {
#pragma unroll
                for (int q = 0; q < PD; ++q)
                    if (q < nq_d) *reinterpret_cast<f4 *>(Dsm + dsbase + q * dsstep) = pd[q];
            }
        } else {
#pragma unroll
            for (int q = 0; q < PI; ++q)
                if (q < nq_in) Ism[isbase + q * isstep] = pin[q];
#pragma unroll
            for (int q = 0; q < PD; ++q)
                if (q < nq_d) Dsm[dsbase + q * dsstep] = pd[q];
        }
    };

    const int xsteps = g.OWP >> 2;
    auto operands = [&](float (&a)[MT], float (&bv)[NTW], int doff, int po) {
#pragma unroll
        for (int m = 0; m < MT; ++m) a[m] = Dsm[ab[m] + doff];
#pragma unroll
        for (int j = 0; j < NTW; ++j) bv[j] = Ism[kb[j] + po];
    };
    auto products = [&](const float (&a)[MT], const float (&bv)[NTW]) {
#pragma unroll
        for (int j = 0; j < NTW; ++j)
#pragma unroll
            for (int m = 0; m < MT; ++m) acc[m][j] = mfma16x16x4(a[m], bv[j], acc[m][j]);
    };

    // The slice's share: output rows u0 .. u1-1 of the client's work items laid end to end (R
    // rows each), so that the shares differ by at most one row; an item cut by a share's end
    // is staged whole by both neighbours and each runs its own rows of it.
    const int u0 = sl * g.U, u1 = min(u0 + g.U, items * g.R);
    int it = u0 / g.R;
    const int it_last = u1 > u0 ? (u1 - 1) / g.R : -1;
    if (it <= it_last) fetch(it);
    for (; it <= it_last; ++it) {
        __syncthreads();   // the products of the previous item are done with the tiles
        stash();
        __syncthreads();
        if (it < it_last) fetch(it + 1);   // in flight while the products run
        const int r_lo = max(u0 - it * g.R, 0), r_hi = min(u1 - it * g.R, g.R);
        const int t_lo = r_lo * xsteps, t_hi = r_hi * xsteps;
        // One step = 4 consecutive pixels of a row.  Two operand sets take turns: the set of
        // the step after is read from LDS before the products of a step are issued.
        float a0[MT], b0[NTW], a1[MT], b1[NTW];
        int xs = 0, po = r_lo * g.SWP;
        auto advance = [&]() {
            po += 4;
            if (++xs == xsteps) { xs = 0; po += g.SWP - g.OWP; }
        };
        operands(a0, b0, 4 * t_lo, po);
        for (int t = t_lo; t < t_hi; t += 2) {
            const bool odd = t + 1 < t_hi;
            if (odd) {
                advance();
                operands(a1, b1, 4 * (t + 1), po);
            }
            products(a0, b0);
            if (t + 2 < t_hi) {
                advance();
                operands(a0, b0, 4 * (t + 2), po);
            }
            if (odd) products(a1, b1);
        }
    }
    // partial[a][slice][co][k]: lane holds k = 16*nt + li, co = 16*mt + 4*lg + r
    const int KP = 16 * g.NTT, OCP = 16 * g.MTT;
    const gf_ptr pg = as_global(partial) + ((int64_t)blockIdx.z * g.S + sl) * OCP * KP;
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
        const int nt = n0 + NS * j;
        if (nt >= g.NTT) continue;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            const int mt = m0 + WM * m;
            if (mt >= g.MTT) continue;
#pragma unroll
            for (int r = 0; r < 4; ++r) pg[(int64_t)(16 * mt + 4 * lg + r) * KP + 16 * nt + li] = acc[m][j][r];
        }
    }
}

// g = (sum of the partials in slice order) / B;  w <- w - eta g;  U <- U + g
__global__ void __launch_bounds__(256)
k_conv_wgrad_finish(const RoundParams *__restrict__ rp, int u, int B, WgradGeom g, int KSQ,
                    const float *__restrict__ partial) {
    const RoundParams p = rp[blockIdx.z];
    if (u >= p.m) return;
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    const int co = blockIdx.y;
    if (k >= g.KTOT) return;
    const int KP = 16 * g.NTT, OCP = 16 * g.MTT;
    const gcf_ptr pg = as_global(partial) + (int64_t)blockIdx.z * g.S * OCP * KP + (int64_t)co * KP + k;
    float s = 0.f;
#pragma unroll 8
    for (int sl = 0; sl < g.S; ++sl) s += pg[(int64_t)sl * OCP * KP];   // loads in flight together, sum in order
    s *= 1.0f / (float)B;
    const int64_t wi = k < g.IC * KSQ ? g.w_off + (int64_t)co * g.IC * KSQ + k : g.b_off + co;
    as_global(p.W)[wi] -= p.eta * s;
    as_global(p.U)[wi] += s;
}

// Workgroups the partial sums of one launch are spread over, at most: layers with a small
// gradient (partial result up to 16 KB) can afford many short slices, which hides the
// latency of their short work items; large ones pay for every slice with a partial result.
static int wgrad_target(const LayerGeom &L) {
    const int64_t floats = (int64_t)((L.oc + 15) / 16 * 16) * ((L.ic * L.k * L.k + 1 + 15) / 16 * 16);
    return floats <= 4096 ? 2048 : 512;
}

// accumulator tiling of the wave: WM = 2 (2 x 2 waves) when there are at most 2 N tiles
static int wgrad_wm(const WgradGeom &g) { return g.NTT <= 2 ? 2 : 1; }
static int wgrad_mt(const WgradGeom &g) {
    const int n = (g.MTT + wgrad_wm(g) - 1) / wgrad_wm(g);
    return n <= 1 ? 1 : n <= 2 ? 2 : 4;
}

static bool wgrad_geom(const LayerGeom &L, int B, int nact, WgradGeom *g) {
    const int KS = L.k;
    if (!(KS == 3 || KS == 5)) return false;
    g->IC = L.ic; g->OC = L.oc; g->IH = L.ih; g->IW = L.iw; g->OH = L.oh; g->OW = L.ow; g->pad = L.pad;
    g->in_size = L.in_size; g->out_size = L.out_size; g->w_off = L.w_off; g->b_off = L.b_off;
    g->KTOT = L.ic * KS * KS + 1;
    g->NTT = (g->KTOT + 15) / 16;
    g->MTT = (L.oc + 15) / 16;
    if (g->MTT > 4 || g->NTT > 40) return false;
    if (L.in_size >= (int64_t)1 << 28 || L.out_size >= (int64_t)1 << 28) return false;   // 32-bit byte offsets
    g->R = L.oh < 4 ? L.oh : 4;
    g->rowsT = g->R + KS - 1;
    g->OWP = (L.ow + 3) / 4 * 4;
    g->SWP = g->OWP + KS - 1;
    g->SWP += (g->SWP & 1) ? 0 : 1;
    g->items_per_sample = (L.oh + g->R - 1) / g->R;
    (void)nact;
    g->S = 1;  // set by the launcher from the number of resident workgroups
    g->U = g->R;
    g->MTS = wgrad_wm(*g) * wgrad_mt(*g);
    g->DPL = g->R * g->OWP + ((4 - (g->R * g->OWP) % 32 + 32) % 32);
    const int plane = g->rowsT * g->SWP, dplane = g->R * g->OWP;
    g->gin = plane <= 256 ? 256 / plane : 0;
    g->gd = dplane <= 256 ? 256 / dplane : 0;
    g->nq_in_all = g->gin ? (g->IC + g->gin - 1) / g->gin : 0;
    g->nq_d_all = g->gd ? (16 * g->MTS + g->gd - 1) / g->gd : 0;
    // four pixels per thread: whole aligned float4s per image row and per d(output) row
    g->vec = 0;
    g->gin4 = g->gd4 = g->nq_in4 = g->nq_d4 = 0;
    if ((L.iw & 3) == 0 && (L.ow & 3) == 0) {
        const int islots = g->rowsT * (L.iw >> 2), dslots = g->R * (L.ow >> 2);
        if (islots <= 256 && dslots <= 256) {
            g->gin4 = 256 / islots;
            g->gd4 = 256 / dslots;
            g->nq_in4 = (g->IC + g->gin4 - 1) / g->gin4;
            g->nq_d4 = (16 * g->MTS + g->gd4 - 1) / g->gd4;
            g->vec = g->nq_in4 <= kPreIn4 && g->nq_d4 <= kPreD4;
        }
    }
    return true;
}

static int wgrad_ntw(const WgradGeom &g) {
    if (wgrad_wm(g) == 2) return 1;
    const int n = (g.NTT + 3) / 4;
    return n <= 2 ? 2 : n <= 5 ? 5 : 10;
}
static size_t wgrad_lds_bytes(const WgradGeom &g) {
    const int CP = g.vec ? g.gin4 * g.nq_in4 : g.gin * g.nq_in_all, DR = g.vec ? g.gd4 * g.nq_d4 : g.gd * g.nq_d_all;
    return sizeof(float) * ((((size_t)(CP + 3) * g.rowsT * g.SWP + 3) & ~(size_t)3) + (size_t)(DR + 1) * g.DPL);
}

bool conv_wgrad_mfma_supported(const LayerGeom &L, int B) {
    WgradGeom g;
    if (!wgrad_geom(L, B, 1, &g)) return false;
    // a thread is tied to one tile position: both tiles must fit the 256 threads, and the
    // channels one thread walks must fit its prefetch registers
    if (g.gin < 1 || g.gd < 1) return false;
    if (g.nq_in_all > kPreIn || g.nq_d_all > kPreD) return false;
    return wgrad_lds_bytes(g) <= 64 * 1024;
}

// floats of partial-sum scratch the layer needs, whatever the number of active clients
size_t conv_wgrad_partial_floats(const LayerGeom &L, int B, int n_clients) {
    WgradGeom g;
    if (!wgrad_geom(L, B, 1, &g)) return 0;
    // nact * S <= wgrad_target + nact
    return (size_t)(wgrad_target(L) + n_clients) * 16 * g.MTT * 16 * g.NTT;
}

// resident workgroups per compute unit of one instantiation (cached); 0 = no such instantiation
template <int KS, int MT, int NTW, int WM, bool VEC>
static int wgrad_blocks_per_cu(size_t lds) {
    static int cached = -1;
    static size_t cached_lds = 0;
    if (cached < 0 || cached_lds != lds) {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_conv_wgrad_mfma<KS, MT, NTW, WM, VEC>, 256, lds) != hipSuccess || n < 1)
            n = 1;
        cached = n;
        cached_lds = lds;
    }
    return cached;
}

// which: 0 = resident workgroups per compute unit, 1 = launch
template <int KS>
static int wgrad_dispatch(int which, hipStream_t s, dim3 grid, size_t lds, int mt, int ntw, int wm,
                          const RoundParams *dp, int u, int B, const WgradGeom &g, const float *in,
                          const float *dout, float *partial) {
#define AET_WG(MTv, NTWv, WMv)                                                                                  \
    if (mt == MTv && ntw == NTWv && wm == WMv) {                                                                \
        if (g.vec) {                                                                                            \
            if (which == 0) return wgrad_blocks_per_cu<KS, MTv, NTWv, WMv, true>(lds);                          \
            k_conv_wgrad_mfma<KS, MTv, NTWv, WMv, true><<<grid, 256, lds, s>>>(dp, u, B, g, in, dout, partial);  \
        } else {                                                                                                \
            if (which == 0) return wgrad_blocks_per_cu<KS, MTv, NTWv, WMv, false>(lds);                         \
            k_conv_wgrad_mfma<KS, MTv, NTWv, WMv, false><<<grid, 256, lds, s>>>(dp, u, B, g, in, dout, partial); \
        }                                                                                                       \
        return 1;                                                                                               \
    }
    AET_WG(1, 1, 2) AET_WG(2, 1, 2)
    AET_WG(1, 2, 1) AET_WG(1, 5, 1) AET_WG(1, 10, 1)
    AET_WG(2, 2, 1) AET_WG(2, 5, 1) AET_WG(2, 10, 1)
    AET_WG(4, 2, 1) AET_WG(4, 5, 1) AET_WG(4, 10, 1)
#undef AET_WG
    return 0;
}


hipError_t launch_conv_wgrad_mfma(hipStream_t s, Profiler *prof, const RoundParams *dp, int nact, int u,
                                  int B, const LayerGeom &L, const float *in, const float *dout,
                                  float *partial) {
    WgradGeom g;
    if (!wgrad_geom(L, B, nact, &g)) return hipErrorInvalidValue;
    const size_t lds = wgrad_lds_bytes(g);
    const int mt = wgrad_mt(g), ntw = wgrad_ntw(g), wm = wgrad_wm(g);
    dim3 none(1, 1, 1);
    const int per_cu = L.k == 3 ? wgrad_dispatch<3>(0, s, none, lds, mt, ntw, wm, dp, u, B, g, in, dout, partial)
                                : wgrad_dispatch<5>(0, s, none, lds, mt, ntw, wm, dp, u, B, g, in, dout, partial);
    if (per_cu < 1) return hipErrorInvalidValue;
    // Slices per client: all workgroups of the launch resident at once (a few workgroups more
    // than fit would cost a whole second pass), never more than the partial-sum scratch holds
    // (wgrad_target + n_clients slices), and the output rows of the work items spread evenly.
    const int units = B * g.items_per_sample * g.R;
    int cap = per_cu * device_cus();
    if (cap > wgrad_target(L)) cap = wgrad_target(L);
    int S = cap / nact;
    if (S < 1) S = 1;
    if (S > units) S = units;
    g.U = (units + S - 1) / S;
    S = (units + g.U - 1) / g.U;  // the fewest slices with the same longest share
    g.S = S;
    const bool timed = prof && prof->on[F_CONV_BWD_WEIGHT];
    if (timed) prof->before(F_CONV_BWD_WEIGHT, s);
    dim3 grid((unsigned)g.S, 1, (unsigned)nact);
    if (L.k == 3) wgrad_dispatch<3>(1, s, grid, lds, mt, ntw, wm, dp, u, B, g, in, dout, partial);
    else wgrad_dispatch<5>(1, s, grid, lds, mt, ntw, wm, dp, u, B, g, in, dout, partial);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) {
        dim3 fgrid((unsigned)((g.KTOT + 255) / 256), (unsigned)g.OC, (unsigned)nact);
        k_conv_wgrad_finish<<<fgrid, 256, 0, s>>>(dp, u, B, g, L.k * L.k, partial);
        e = hipGetLastError();
    }
    if (timed) prof->after(F_CONV_BWD_WEIGHT, s);
    return e;
}

}  // namespace aet
