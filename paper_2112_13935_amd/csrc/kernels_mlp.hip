// Fused local round for dense-ReLU-dense models (D -> H -> C, mini-batch B = 16 or 32).
//
// One launch runs the whole round (Algorithm 2, MainComputeNode: all s_i/B recursions) of
// every active client.  A client is handled by a cluster of G = H/16 workgroups; workgroup
// g owns hidden units 16g..16g+15: its slice of the first layer (16 x D weights, 16
// biases) and of the second layer (C x 16 weights), together with the matching slices of
// U, stay in registers / LDS for the whole round, so the per-recursion traffic is the
// mini-batch rows plus one small exchange.
//
// Per recursion:
//   - each of the 8 waves owns a contiguous eighth of the input columns: it has loaded its
//     part of the B sampled rows into registers during the previous recursion, in the
//     A-operand layout of the forward product;
//   - z1 = X W1^T on the matrix cores (fp32 MFMA 16x16x4) straight from those registers,
//     partial over the wave's columns, summed over the waves through LDS; h = relu(z1 + b1);
//     the rows are then parked in LDS for the backward product (no workgroup barrier:
//     nobody else touches those columns);
//   - the partial logits of the 16 own units are written to the client's exchange record
//     as 64-bit {step tag, value} words; every workgroup polls the G records until all
//     tags show the current step, which gives the logits without a separate barrier or
//     fence (each word validates itself; two records alternate so a fast workgroup never
//     overwrites what a slow one still has to read);
//   - softmax / d logits with 16 lanes per sample; dh = (d logits W2) * 1[h > 0] and
//     dW2 = d logits^T h as small MFMA products;
//   - dW1^T = X^T dh on the matrix cores: the accumulator tile has exactly the register
//     layout the forward pass uses as its B operand, so  w <- w - eta g  and  U <- U + g
//     are applied to the register-resident slice in place (g never exists in memory).
//
// Wide inputs (more than 32 column tiles) with few enough clients take two workgroups per
// unit group: each owns half of the input columns (its half of the W1 / U1 slice, of the
// sampled rows, of the forward and of the backward product); the two add their partial
// hidden sums through a second tagged exchange and then compute the same h, logits and
// second-layer updates side by side.  16 clients x 8 unit groups then occupy all 256
// compute units instead of 128.
//
// All workgroups of a client must be resident together: the launcher never has more
// working workgroups in flight than the device holds (1 per compute unit with this LDS
// footprint).  The poll is bounded: on expiry an error flag is raised and every workgroup
// still runs to the end, so the grid always drains.
#include "aet_device.h"
#include "aet_internal.h"

namespace aet {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kMlpWaves = 8;         // waves per workgroup (2 per SIMD)
constexpr int kMlpThreads = 64 * kMlpWaves;
constexpr int kMlpMaxTPW = 7;        // K tiles (of 16) per wave  => D <= 16*8*7 = 896
constexpr int kMlpMaxG = 16;         // workgroups per client
constexpr int kMlpRec = 512;         // 64-bit words per exchange record (B*C <= 512)
constexpr int kMlpPair = 512;        // 64-bit words per pair record (B*16 <= 512)
constexpr int kMlpHalfTPW = 4;       // K tiles per wave when two workgroups share the columns
constexpr int kSpinLimit = 1 << 22;  // bounded wait of the exchange poll

// Hides a value from the optimiser so that addresses derived from it are computed where
// they are used instead of being kept in registers across the whole recursion loop.
__device__ __forceinline__ int opaque(int x) {
    asm volatile("" : "+v"(x));
    return x;
}

__device__ __forceinline__ f4 mfma16(float a, float b, f4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}
// sum / max over the 16 lanes of one sample (lanes 16k .. 16k+15 of the wave), with the
// data-parallel-primitive lane permutations inside a row: neighbours in a quad, the other
// pair of the quad, the mirrored half row, the mirrored row
#define AET_ROW_STEP(op, v, ctrl) \
    v = op(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), ctrl, 0xF, 0xF, true)))
__device__ __forceinline__ float row16_add(float a, float b) { return a + b; }
__device__ __forceinline__ float row16_sum(float v) {
    AET_ROW_STEP(row16_add, v, 0xB1);
    AET_ROW_STEP(row16_add, v, 0x4E);
    AET_ROW_STEP(row16_add, v, 0x141);
    AET_ROW_STEP(row16_add, v, 0x140);
    return v;
}
__device__ __forceinline__ float row16_max(float v) {
    AET_ROW_STEP(fmaxf, v, 0xB1);
    AET_ROW_STEP(fmaxf, v, 0x4E);
    AET_ROW_STEP(fmaxf, v, 0x141);
    AET_ROW_STEP(fmaxf, v, 0x140);
    return v;
}
#undef AET_ROW_STEP

// sum over the 64 lanes, every lane gets it (gfx950 lane swaps: halves, then rows, then the
// in-row steps)
__device__ __forceinline__ float fold_rows(float v) {   // sum of the 4 rows, lane by lane
    const auto a = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(int, v), __builtin_bit_cast(int, v), false, false);
    v = __builtin_bit_cast(float, (int)a[0]) + __builtin_bit_cast(float, (int)a[1]);
    const auto b = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(int, v), __builtin_bit_cast(int, v), false, false);
    return __builtin_bit_cast(float, (int)b[0]) + __builtin_bit_cast(float, (int)b[1]);
}
// column sums of a [B][16] LDS array: lane (c = lane % 16, q = lane / 16) adds the rows
// q, q + 4, ... of column c, then the four row groups are folded
template <int B>
__device__ __forceinline__ float col_sum16(const float *a, int lane) {
    float s = 0.f;
#pragma unroll
    for (int b = lane >> 4; b < B; b += 4) s += a[b * 16 + (lane & 15)];
    return fold_rows(s);
}

// FAST: D is a multiple of 16, so every row piece is one aligned 16-byte load.
// NBT: batch tiles of 16 samples; TPW: K-tile slots of a wave (a wave that owns fewer tiles
// skips the rest with scalar branches).
// The round records of one launch travel in the kernel arguments: no staging copy, no
// buffer whose reuse would have to be fenced with events.
constexpr int kMlpPack = 48;
struct MlpPack {
    RoundParams p[kMlpPack];
};

// FULL: every wave owns TPW real tiles (D = 16 * 8 * TPW): no pad tiles, loads unguarded.
// HF = 2: two workgroups per unit group, each owning one half of the input columns (its
// half of the W1 / U1 slice, of the sampled rows and of both big products); they add their
// partial hidden sums through a second tagged exchange (pair records `prec`) and from
// there on compute the same numbers side by side; half 0 posts the logits and stores the
// second layer at the end.
template <int NBT, int TPW, bool FAST, bool FULL, int HF>
__global__ void __launch_bounds__(kMlpThreads, 1)
k_mlp_round(const MlpPack pack, int nhere, int rec0, const float *Wg,
            int D, int H, int C, int G, unsigned long long *__restrict__ xrec,
            unsigned long long *__restrict__ prec, uint32_t tag0, int *__restrict__ errflag) {
    constexpr int B = 16 * NBT;
    // workgroup -> (client, unit group, half): consecutive workgroup ids go round the 8 XCDs,
    // so the workgroups of one client get ids that land on the same XCD and share its L2
    // for the mini-batch rows and the exchanges.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int a = xcd + 8 * (slot / (G * HF));  // index into this launch's records
    const int g = (slot % (G * HF)) / HF, hf = slot % HF;
    if (a >= nhere) return;
    const RoundParams p = pack.p[a];
    const gcf_ptr Xg = as_global(p.X);
    const gci_ptr yg = as_global(p.y);
    const gf_ptr Wc = as_global(p.W), Uc = as_global(p.U);

    const int tid = threadIdx.x, lane = tid & 63, li = lane & 15, lg = lane >> 4;
    // the wave index as a scalar, so that everything derived from it (tile counts, column
    // offsets, branches on them) stays in scalar registers and scalar branches
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // real K tiles (of 16 columns) of this half, and the first of them
    const int KTall = (D + 15) >> 4, KH = (KTall + HF - 1) / HF;
    const int tbase = hf * KH;
    const int KT = min(KH, KTall - tbase);
    constexpr int ld = 16 * kMlpWaves * TPW + 4;  // LDS row stride: all tiles + 4 floats of skew
    constexpr int NI = NBT * TPW;             // float4 loads per lane and mini-batch
    // the KT tiles are dealt out evenly: wave w owns nt consecutive tiles from t0 on, the
    // first KT % 8 waves one more than the others (waves w and w + 4 share a SIMD and its
    // matrix core: dealt this way the four SIMDs differ by one tile at most).  A wave has
    // TPW tile slots in registers and in the staged rows; slots beyond nt are skipped.
    const int tb = KT / kMlpWaves, te = KT % kMlpWaves;
    const int nt = tb + (wave < te ? 1 : 0);
    const int t0 = wave * tb + min(wave, te);
    const int col0 = 16 * TPW * wave;         // first column of the wave's slots in the staged rows
    const int gcol0 = 16 * (tbase + t0);      // first own column in the sample / weight rows

    extern __shared__ float smem[];
    // the small arrays come first so that their addresses fit the 16-bit offset field of
    // the LDS instructions; the big mini-batch tile follows
    float *red = smem;                // [waves][B][16]
    float *hs = red + kMlpWaves * B * 16;  // [B][16]
    float *dhs = hs + B * 16;         // [B][16]
    float *zs = dhs + B * 16;         // [B][16]  d logits (columns >= C stay 0)
    float *W2s = zs + B * 16;         // [16][16] (o, j)
    float *U2s = W2s + 256;
    float *b1s = U2s + 256;           // [16]
    float *Ub1s = b1s + 16;
    float *b2s = Ub1s + 16;
    float *Ub2s = b2s + 16;
    float *lossb = Ub2s + 16;         // [B]
    float *lossacc = lossb + B;       // [16], entry 0: the round's loss sum
    int *labs = reinterpret_cast<int *>(lossacc + 16);  // [B]
    float *Xs = reinterpret_cast<float *>(labs + B); // [B][ld]

    const int64_t b1_off = (int64_t)H * D, w2_off = b1_off + H, b2_off = w2_off + (int64_t)C * H;
    const float invB = 1.0f / (float)B;

    // The mini-batch travels global -> registers -> matrix core / LDS in the A-operand layout
    // of the forward product: lane (li, lg) holds, for batch tile bt and K tile tt, the four
    // values x[16*bt + li][col0 + 16*tt + 4*lg .. +3] (one 16-byte load when FAST: D a
    // multiple of 16, so every piece is inside the row and aligned).
    const gcf_ptr lane_src = Xg + gcol0 + 4 * lg;
    // rowp: the lane's piece of tile 0 of its row, lane_src + row * D
    auto load_piece = [&](gcf_ptr rowp, int tt) -> f4 {
        f4 x = {0.f, 0.f, 0.f, 0.f};
        if (FULL || tt < nt) {
            const gcf_ptr src = rowp + 16 * tt;
            if constexpr (FAST) {
                x = *reinterpret_cast<const f4 __attribute__((address_space(1))) *>(src);
            } else {
                const int col = gcol0 + 16 * tt + 4 * lg;
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (col + r < D) x[r] = src[r];
            }
        }
        return x;
    };

    // ---- adopt the global model (server form) or go on from the own replica (Wg == NULL:
    // peer-to-peer form): own slice into registers / LDS; U = 0 -------------------------
    if (!Wg) Wg = p.W;
    f4 W1r[TPW], U1r[TPW];
#pragma unroll
    for (int tt = 0; tt < TPW; ++tt) {
        f4 w = {0.f, 0.f, 0.f, 0.f};
        if (tt < nt) {
            const float *src = Wg + (int64_t)(16 * g + li) * D + gcol0 + 16 * tt + 4 * lg;
            if constexpr (FAST) {   // D a multiple of 16: the four values are one aligned piece
                w = *reinterpret_cast<const f4 *>(src);
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (gcol0 + 16 * tt + 4 * lg + r < D) w[r] = src[r];
            }
        }
        W1r[tt] = w;
        U1r[tt] = f4{0.f, 0.f, 0.f, 0.f};
    }
    {
        const int o = tid >> 4, j = tid & 15;  // threads 0..255 = 16 x 16
        if (tid < 256) {
            W2s[tid] = (o < C) ? Wg[w2_off + (int64_t)o * H + 16 * g + j] : 0.f;
            U2s[tid] = 0.f;
        }
        for (int i = tid; i < B * 16; i += kMlpThreads) zs[i] = 0.f;
        if (tid < 16) {
            b1s[tid] = Wg[b1_off + 16 * g + tid];
            Ub1s[tid] = 0.f;
            b2s[tid] = (tid < C) ? Wg[b2_off + tid] : 0.f;
            Ub2s[tid] = 0.f;
            lossacc[tid] = 0.f;
        }
    }
    __syncthreads();
    // rows of recursion 0 into registers, labels into LDS
    f4 xreg[NBT][TPW];
#pragma unroll
    for (int bt = 0; bt < NBT; ++bt)
#pragma unroll
        for (int tt = 0; tt < TPW; ++tt) xreg[bt][tt] = f4{0.f, 0.f, 0.f, 0.f};
    if (p.m > 0) {
        uint32_t rowv = 0;
        if (lane < B) rowv = sample_row(p.key, (uint64_t)(p.q0 + lane), p.n_samples);
        if (wave == 0 && lane < B) labs[lane] = yg[rowv];
#pragma unroll
        for (int bt = 0; bt < NBT; ++bt) {
            const gcf_ptr rowp = lane_src + (int64_t)__shfl(rowv, 16 * bt + li) * D;
#pragma unroll
            for (int tt = 0; tt < TPW; ++tt) xreg[bt][tt] = load_piece(rowp, tt);
        }
    }
    unsigned long long *rec_base = xrec + (int64_t)(rec0 + a) * 2 * kMlpMaxG * kMlpRec;
    // pair records [client][unit group][step parity][half][B * 16]
    unsigned long long *prec_base = prec + ((int64_t)(rec0 + a) * kMlpMaxG + g) * 4 * kMlpPair;
    bool dead = false;  // the poll expired: keep going, the host will see the flag
    __syncthreads();

    auto park_rows = [&]() {
#pragma unroll
        for (int bt = 0; bt < NBT; ++bt)
#pragma unroll
            for (int tt = 0; tt < TPW; ++tt)
                if (FULL || tt < nt)
                    *reinterpret_cast<f4 *>(Xs + (16 * bt + li) * ld + col0 + 16 * tt + 4 * lg) = xreg[bt][tt];
    };
    for (int u = 0; u < p.m; ++u) {
        // ---- z1 partial sums on the matrix cores ----------------------------------------
        {
            f4 acc[NBT];
#pragma unroll
            for (int bt = 0; bt < NBT; ++bt) acc[bt] = f4{0.f, 0.f, 0.f, 0.f};
            // the A operand comes straight from the registers the rows were loaded into
            // (all TPW slots, free of branches: an empty slot holds zeros on both sides; skipping
            // it measured slower here, while the backward product below gains from skipping)
#pragma unroll
            for (int tt = 0; tt < TPW; ++tt) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int bt = 0; bt < NBT; ++bt) acc[bt] = mfma16(xreg[bt][tt][r], W1r[tt][r], acc[bt]);
            }
            // the backward product needs the rows transposed: park them in LDS (this wave's
            // columns only, so no barrier; the writes drain while the logits are exchanged).
            // With two workgroups per unit group they are parked between the post and the
            // poll of the pair exchange instead.
            if constexpr (HF == 1) park_rows();
#pragma unroll
            for (int bt = 0; bt < NBT; ++bt)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    red[(wave * B + 16 * bt + 4 * lg + r) * 16 + li] = acc[bt][r];
        }
        __syncthreads();
        // the rows the next recursion samples (Algorithm 2, sampling step; a counter
        // hash, so they are known ahead); with two workgroups per unit group the hash is
        // computed while the pair exchange is in flight
        uint32_t rowv = 0;
        const bool more = u + 1 < p.m;
        auto next_rows = [&]() {
            if (more && lane < B) rowv = sample_row(p.key, (uint64_t)(p.q0 + (int64_t)(u + 1) * B + lane), p.n_samples);
        };
        // ---- h = relu(z1 + b1) ----------------------------------------------------------
        const uint32_t tag = tag0 + (uint32_t)u;
        if constexpr (HF == 1) {
            for (int i = tid; i < B * 16; i += kMlpThreads) {
                float s = b1s[i & 15];
#pragma unroll
                for (int w = 0; w < kMlpWaves; ++w) s += red[w * B * 16 + i];
                hs[i] = s > 0.f ? s : 0.f;
            }
        } else {
            // the own half's sums go to the pair record, the other half's come from there;
            // both halves add them in the same order (half 0 + half 1), so both get the same h
            unsigned long long *pr = prec_base + (int64_t)(u & 1) * 2 * kMlpPair;
            const int i = tid;   // B * 16 <= 512 elements, one per thread
            float own = 0.f;
            if (i < B * 16) {
#pragma unroll
                for (int w = 0; w < kMlpWaves; ++w) own += red[w * B * 16 + i];
                const unsigned long long word = ((unsigned long long)tag << 32) | (unsigned long long)__float_as_uint(own);
                __hip_atomic_store(pr + hf * kMlpPair + i, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            park_rows();
            next_rows();
            const unsigned long long *theirs = pr + (1 - hf) * kMlpPair + min(i, B * 16 - 1);
            unsigned long long v = 0;
            int spins = 0;
            for (;;) {
                v = __hip_atomic_load(theirs, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (__all((uint32_t)(v >> 32) == tag) || dead) break;
                __builtin_amdgcn_s_sleep(1);
                if ((++spins & 255) == 0) {
                    if (spins >= kSpinLimit || __hip_atomic_load(errflag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                        __hip_atomic_store(errflag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        dead = true;
                    }
                }
            }
            if (i < B * 16) {
                const float other = __uint_as_float((uint32_t)v);
                const float s = b1s[i & 15] + (hf == 0 ? own + other : other + own);
                hs[i] = s > 0.f ? s : 0.f;
            }
        }
        __syncthreads();
        // ---- partial logits of the own 16 units -> tagged exchange record ---------------
        unsigned long long *rec = rec_base + (int64_t)(u & 1) * kMlpMaxG * kMlpRec;
        if (wave < NBT && hf == 0) {
            const int bt = wave;
            f4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s)
                acc = mfma16(hs[(16 * bt + li) * 16 + 4 * s + lg], W2s[li * 16 + 4 * s + lg], acc);
            if (li < C) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int b = 16 * bt + 4 * lg + r;
                    const unsigned long long word = ((unsigned long long)tag << 32) | (unsigned long long)__float_as_uint(acc[r]);
                    __hip_atomic_store(rec + (int64_t)g * kMlpRec + b * C + li, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
        // ---- prefetch the rows of the NEXT recursion into registers ----------------------
        // (Algorithm 2, sampling step; the indices are a counter hash, so they are
        // known ahead of time).  Loads of one wave return in order, so nothing is issued
        // before the exchange poll.
        int labn = 0;
        // the rows' indices and the labels now; the row loads themselves are issued a few at
        // a time between the first tiles of the backward product, so that a wave that has to
        // wait for room in the memory pipeline leaves the matrix core to the SIMD's other
        // wave.  They go into the registers the forward product has finished with.
        gcf_ptr myrow[NBT];
        auto prefetch_rows = [&]() {
            if (!more) return;
            if constexpr (HF == 1) next_rows();
            if (wave == 0 && lane < B) labn = yg[rowv];
#pragma unroll
            for (int bt = 0; bt < NBT; ++bt) myrow[bt] = lane_src + (int64_t)__shfl(rowv, 16 * bt + li) * D;
        };
        constexpr int PFT = TPW > 4 ? 4 : TPW;   // tiles of the backward product that carry loads
        auto prefetch_load = [&](int i) {        // i = tt * NBT + bt: in the order the forward product uses them
            if (!more) return;
            xreg[i % NBT][i / NBT] = load_piece(myrow[i % NBT], i / NBT);
        };
        // ---- logits, softmax, d logits: thread (b, o) = (tid / 16, tid % 16) ------------
        // Every thread with o < C fetches its own logit: the G tagged words of element
        // (b, o).  Polling loads slow the peers' stores down (they meet in the same memory
        // channels: a variant in which every thread polls its own words ran a quarter slower), so
        // while the peers are still computing only wave 0 looks, and only at one word per
        // record and batch tile (the last one its owner stores); the other waves wait at a
        // workgroup barrier.  The elements are fetched when those words show the current tag;
        // the element tags are still checked, and the fetch repeated if one is stale.  (A
        // separate flag word per poster, stored after the logits, overtakes them on the way
        // and makes the fetch fail: the watched word has to be one of the data words.)
        {
            const int b = tid >> 4, o = tid & 15;
            const bool mine = b < B && o < C;
            float z = 0.f;
            int spins = 0;
            if (wave == 0) {
                // lane -> (record, batch tile); the word of sample 16*bt+15, class C-1
                const int gg = lane % G, bt = lane / G;
                const bool watch = bt < NBT;
                const unsigned long long *w = rec + (int64_t)gg * kMlpRec + (16 * min(bt, NBT - 1) + 15) * C + (C - 1);
                for (;;) {
                    bool ok = true;
                    if (watch) ok = (uint32_t)(__hip_atomic_load(w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >> 32) == tag;
                    if (__all(ok) || dead) break;
                    __builtin_amdgcn_s_sleep(2);
                    if ((++spins & 255) == 0) {
                        if (spins >= kSpinLimit || __hip_atomic_load(errflag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                            __hip_atomic_store(errflag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            dead = true;
                        }
                    }
                }
            }
            __syncthreads();
            if (mine) {
                const unsigned long long *src = rec + b * C + o;
                constexpr int GC = 8;  // records fetched per batch of loads
                for (;;) {
                    bool ok = true;
                    z = b2s[o];
                    if (G == GC) {   // the common cluster size: one unguarded batch
                        unsigned long long v[GC];
#pragma unroll
                        for (int gg = 0; gg < GC; ++gg)
                            v[gg] = __hip_atomic_load(src + gg * kMlpRec, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                        for (int gg = 0; gg < GC; ++gg) {
                            ok = ok && (uint32_t)(v[gg] >> 32) == tag;
                            z += __uint_as_float((uint32_t)v[gg]);
                        }
                    } else {
                        for (int g0 = 0; g0 < G; g0 += GC) {
                            unsigned long long v[GC];
#pragma unroll
                            for (int gg = 0; gg < GC; ++gg)
                                if (g0 + gg < G) v[gg] = __hip_atomic_load(src + (g0 + gg) * kMlpRec, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                            for (int gg = 0; gg < GC; ++gg)
                                if (g0 + gg < G) {
                                    ok = ok && (uint32_t)(v[gg] >> 32) == tag;
                                    z += __uint_as_float((uint32_t)v[gg]);
                                }
                        }
                    }
                    if (ok || dead) break;
                    __builtin_amdgcn_s_sleep(2);
                    if ((++spins & 255) == 0) {
                        if (spins >= kSpinLimit || __hip_atomic_load(errflag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                            __hip_atomic_store(errflag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            dead = true;
                        }
                    }
                }
            }
            if (b < B) {
                const float zmax = row16_max(o < C ? z : -3.0e38f);
                const float ex = o < C ? __expf(z - zmax) : 0.f;
                const float lse = zmax + __logf(row16_sum(ex));
                const int lab = labs[b];
                if (o == lab) lossb[b] = lse - z;
                zs[b * 16 + o] = o < C ? __expf(z - lse) - (o == lab ? 1.f : 0.f) : 0.f;
            }
        }
        __syncthreads();
        // ---- small products on the matrix cores -----------------------------------------
        prefetch_rows();
        f4 dW2acc = {0.f, 0.f, 0.f, 0.f};
        if (wave < NBT) {
            // dh = (dz W2) * 1[h > 0] for samples 16*wave .. 16*wave+15
            const int bt = wave;
            f4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s)
                acc = mfma16(zs[(16 * bt + li) * 16 + 4 * s + lg], W2s[(4 * s + lg) * 16 + li], acc);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int i = (16 * bt + 4 * lg + r) * 16 + li;
                dhs[i] = hs[i] > 0.f ? acc[r] : 0.f;
            }
        } else if (wave == 2) {
            // dW2[o][j] = sum_b dz[b][o] h[b][j]; applied after the barrier (W2 is still read)
#pragma unroll
            for (int s = 0; s < 4 * NBT; ++s)
                dW2acc = mfma16(zs[(4 * s + lg) * 16 + li], hs[(4 * s + lg) * 16 + li], dW2acc);
        } else if (wave == 3) {
            // second-layer bias: column sums of dz
            const float s = col_sum16<B>(zs, lane) * invB;
            if (lane < C) {
                b2s[lane] -= p.eta * s;
                Ub2s[lane] += s;
            }
        } else if (wave == 4) {
            // the recursion's mean loss
            const float s = row16_sum(fold_rows(lane < B ? lossb[lane] : 0.f));
            if (lane == 0) lossacc[0] += s * invB;
        }
        __syncthreads();
        // ---- second layer and first-layer bias: w <- w - eta g, U <- U + g ---------------
        if (wave == 2) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int i = (4 * lg + r) * 16 + li;  // (o, j)
                const float gv = dW2acc[r] * invB;
                W2s[i] -= p.eta * gv;
                U2s[i] += gv;
            }
        } else if (wave == 3) {
            // first-layer bias: column sums of dh
            const float s = col_sum16<B>(dhs, lane) * invB;
            if (lane < 16) {
                b1s[lane] -= p.eta * s;
                Ub1s[lane] += s;
            }
        }
        // ---- first layer: dW1^T = X^T dh on the matrix cores, update in registers -------
        {
            // contraction step s of lane group lg takes sample 16*(s/4) + (s%4) + 4*lg: with
            // rows 4*lg apart the four lane groups read LDS banks 16 apart (ld = 4 mod 32)
            float dhb[4 * NBT];
#pragma unroll
            for (int s = 0; s < 4 * NBT; ++s) dhb[s] = dhs[(16 * (s >> 2) + (s & 3) + 4 * lg) * 16 + li];
            float xb[2][4 * NBT];
            const float *xcol = Xs + opaque(4 * lg * ld + col0 + li);
            if (FULL || nt > 0) {
#pragma unroll
                for (int s = 0; s < 4 * NBT; ++s) xb[0][s] = xcol[(16 * (s >> 2) + (s & 3)) * ld];
            }
            const float eb = p.eta * invB;
#pragma unroll
            for (int tt = 0; tt < TPW; ++tt) {
                if (tt + 1 < TPW && (FULL || tt + 1 < nt)) {
#pragma unroll
                    for (int s = 0; s < 4 * NBT; ++s) xb[(tt + 1) & 1][s] = xcol[(16 * (s >> 2) + (s & 3)) * ld + 16 * (tt + 1)];
                }
                __builtin_amdgcn_sched_barrier(0);   // the next tile's operands are on their way before the products
                if (FULL || tt < nt) {
                    // two independent accumulation chains per tile
                    // (the first product of each chain takes the constant zero as its addend)
                    f4 acc0 = mfma16(xb[tt & 1][0], dhb[0], f4{0.f, 0.f, 0.f, 0.f});
                    f4 acc1 = mfma16(xb[tt & 1][1], dhb[1], f4{0.f, 0.f, 0.f, 0.f});
#pragma unroll
                    for (int s = 2; s < 4 * NBT; s += 2) {
                        acc0 = mfma16(xb[tt & 1][s], dhb[s], acc0);
                        acc1 = mfma16(xb[tt & 1][s + 1], dhb[s + 1], acc1);
                    }
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float gsum = acc0[r] + acc1[r];
                        W1r[tt][r] -= eb * gsum;
                        U1r[tt][r] += invB * gsum;
                    }
                }
                // this tile's share of the next recursion's row loads
#pragma unroll
                for (int i = tt * NI / PFT; i < (tt + 1) * NI / PFT && i < NI; ++i) prefetch_load(i);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // ---- the next recursion's labels ----------------------------------------------------
        if (more && wave == 0 && lane < B) labs[lane] = labn;
    }

    // ---- end of round: the replica and the message payload go to HBM ---------------------
#pragma unroll
    for (int tt = 0; tt < TPW; ++tt) {
        if (tt < nt) {
            const int64_t base = (int64_t)(16 * g + li) * D + gcol0 + 16 * tt + 4 * lg;
            if constexpr (FAST) {
                *reinterpret_cast<f4 __attribute__((address_space(1))) *>(Wc + base) = W1r[tt];
                *reinterpret_cast<f4 __attribute__((address_space(1))) *>(Uc + base) = U1r[tt];
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (gcol0 + 16 * tt + 4 * lg + r < D) {
                        Wc[base + r] = W1r[tt][r];
                        Uc[base + r] = U1r[tt][r];
                    }
            }
        }
    }
    __syncthreads();
    if (hf == 0) {
        const int o = tid >> 4, j = tid & 15;
        if (tid < 256 && o < C) {
            Wc[w2_off + (int64_t)o * H + 16 * g + j] = W2s[tid];
            Uc[w2_off + (int64_t)o * H + 16 * g + j] = U2s[tid];
        }
        if (tid < 16) {
            Wc[b1_off + 16 * g + tid] = b1s[tid];
            Uc[b1_off + 16 * g + tid] = Ub1s[tid];
            if (g == 0 && tid < C) {
                Wc[b2_off + tid] = b2s[tid];
                Uc[b2_off + tid] = Ub2s[tid];
            }
        }
    }
    // the loss was accumulated by wave 4, lane 0 of unit group 0
    if (g == 0 && hf == 0 && wave == 4 && lane == 0) *as_global(p.loss) = lossacc[0];
}

__global__ void k_zero_words(unsigned long long *p, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0ull;
}

static int mlp_tpw(int D) { return (D + 15) / 16 <= 2 * kMlpWaves ? 2 : kMlpMaxTPW; }

static size_t mlp_lds_bytes_tpw(int tpw, int B) {
    const int ld = 16 * kMlpWaves * tpw + 4;
    return sizeof(float) * ((size_t)B * ld + kMlpWaves * B * 16 + 3 * B * 16 + 512 + 64 + B + 16) + sizeof(int) * B;
}
static size_t mlp_lds_bytes(int D, int B) { return mlp_lds_bytes_tpw(mlp_tpw(D), B); }

bool mlp_round_supported(int D, int H, int C, int B) {
    if (!(B == 16 || B == 32)) return false;
    if (H % 16 || H / 16 > kMlpMaxG || C < 1 || C > 16) return false;
    if (D < 1 || (D + 15) / 16 > kMlpWaves * kMlpMaxTPW) return false;
    return mlp_lds_bytes(D, B) <= 160 * 1024;
}

// exchange records [client][2][kMlpMaxG][kMlpRec] 64-bit words, the pair records
// [client][kMlpMaxG][2][2][kMlpPair], then the error flag
static size_t mlp_rec_words(int n_clients) { return (size_t)n_clients * 2 * kMlpMaxG * kMlpRec; }
static size_t mlp_all_words(int n_clients) { return mlp_rec_words(n_clients) + (size_t)n_clients * kMlpMaxG * 4 * kMlpPair; }

size_t mlp_round_scratch_bytes(int n_clients, int B) {
    (void)B;
    return mlp_all_words(n_clients) * 8 + 256;
}

static int g_mlp_capacity[2][3][3] = {};  // resident workgroups, per instantiation

template <int NBT, int TPW, bool FAST, bool FULL, int HF>
static hipError_t mlp_capacity(size_t lds, int *cap) {
    int &cached = g_mlp_capacity[NBT - 1][HF == 2 ? 2 : TPW == kMlpMaxTPW ? 1 : 0][FAST ? (FULL ? 2 : 1) : 0];
    if (cached > 0) { *cap = cached; return hipSuccess; }
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_mlp_round<NBT, TPW, FAST, FULL, HF>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    int dev = 0, cus = 0, per_cu = 0;
    e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_mlp_round<NBT, TPW, FAST, FULL, HF>, kMlpThreads, lds);
    if (e != hipSuccess) return e;
    *cap = cus * per_cu;
    cached = *cap;
    return hipSuccess;
}

// HF = 2 (two workgroups per unit group) is taken only when all active clients fit one
// launch that way; otherwise *declined is set and nothing is launched.
template <int NBT, int TPW, bool FAST, bool FULL, int HF>
static hipError_t mlp_launch(hipStream_t s, Profiler *prof, const RoundParams *hp, int nact, int max_m,
                             const float *Wg, int D, int H, int C, void *scratch, int n_clients,
                             uint32_t *epoch, bool *declined = nullptr) {
    constexpr int B = 16 * NBT;
    const int G = H / 16;
    const size_t lds = mlp_lds_bytes_tpw(TPW, B);
    int cap = 0;
    hipError_t e = mlp_capacity<NBT, TPW, FAST, FULL, HF>(lds, &cap);
    if (e != hipSuccess) return e;
    // Clusters per launch: every workgroup that polls must be resident together with its
    // peers.  Workgroups of unused slots exit at once and free their compute unit, so only
    // the working ones count.
    const int per_launch = cap / (G * HF) < kMlpPack ? cap / (G * HF) : kMlpPack;
    if (HF == 2 && per_launch < nact) {
        *declined = true;
        return hipSuccess;
    }
    if (per_launch < 1) return hipErrorLaunchOutOfResources;
    unsigned long long *xrec = static_cast<unsigned long long *>(scratch);
    unsigned long long *prec = xrec + mlp_rec_words(n_clients);
    int *errflag = reinterpret_cast<int *>(xrec + mlp_all_words(n_clients));
    // step tags of this launch: never 0 (the cleared state) and never a tag that an
    // earlier launch may have left in the records
    if (*epoch == 0 || *epoch > 0xFFFFFFFFu - (uint32_t)max_m - 2u) {
        k_zero_words<<<(unsigned)((mlp_all_words(n_clients) + 255) / 256), 256, 0, s>>>(xrec, mlp_all_words(n_clients));
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        *epoch = 1;
    }
    const uint32_t tag0 = *epoch;
    *epoch += (uint32_t)max_m + 1u;
    for (int a0 = 0; a0 < nact; a0 += per_launch) {
        const int here = (nact - a0 < per_launch) ? nact - a0 : per_launch;
        const int groups = (here + 7) / 8;  // clients per XCD in this launch
        const unsigned grid = (unsigned)(8 * groups * G * HF);
        MlpPack pack;
        for (int j = 0; j < here; ++j) pack.p[j] = hp[a0 + j];
        if (prof && prof->on[F_MLP_ROUND]) prof->before(F_MLP_ROUND, s);
        k_mlp_round<NBT, TPW, FAST, FULL, HF><<<grid, kMlpThreads, lds, s>>>(pack, here, a0, Wg, D, H, C, G, xrec, prec, tag0, errflag);
        if (prof && prof->on[F_MLP_ROUND]) prof->after(F_MLP_ROUND, s);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_mlp_round(hipStream_t s, Profiler *prof, const RoundParams *hp, int nact, int max_m,
                            const float *Wg, int D, int H, int C, int B, void *scratch,
                            int n_clients, uint32_t *epoch) {
    if (nact <= 0) return hipSuccess;
    const bool small = mlp_tpw(D) == 2;  // at most 2 K tiles per wave
    const bool fast = (D & 15) == 0;
    const bool full = D == 16 * kMlpWaves * mlp_tpw(D);   // no pad tiles
    // wide inputs: two workgroups per unit group, half of the columns each, when every active
    // client gets its 2 G workgroups resident in one launch
    if (!small && ((D + 15) / 16 + 1) / 2 <= kMlpWaves * kMlpHalfTPW) {
        bool declined = false;
        hipError_t e;
        if (B == 16) e = fast ? mlp_launch<1, kMlpHalfTPW, true, false, 2>(s, prof, hp, nact, max_m, Wg, D, H, C, scratch, n_clients, epoch, &declined)
                              : mlp_launch<1, kMlpHalfTPW, false, false, 2>(s, prof, hp, nact, max_m, Wg, D, H, C, scratch, n_clients, epoch, &declined);
        else e = fast ? mlp_launch<2, kMlpHalfTPW, true, false, 2>(s, prof, hp, nact, max_m, Wg, D, H, C, scratch, n_clients, epoch, &declined)
                      : mlp_launch<2, kMlpHalfTPW, false, false, 2>(s, prof, hp, nact, max_m, Wg, D, H, C, scratch, n_clients, epoch, &declined);
        if (e != hipSuccess || !declined) return e;
    }
#define AET_MLP_CASE(nbt, tpw)                                                                        \
    do {                                                                                              \
        if (full) return mlp_launch<nbt, tpw, true, true, 1>(s, prof, hp, nact, max_m, Wg, D, H, C, scratch, n_clients, epoch);   \
        if (fast) return mlp_launch<nbt, tpw, true, false, 1>(s, prof, hp, nact, max_m, Wg, D, H, C, scratch, n_clients, epoch);  \
        return mlp_launch<nbt, tpw, false, false, 1>(s, prof, hp, nact, max_m, Wg, D, H, C, scratch, n_clients, epoch);           \
    } while (0)
    if (B == 16) {
        if (small) AET_MLP_CASE(1, 2);
        AET_MLP_CASE(1, kMlpMaxTPW);
    }
    if (small) AET_MLP_CASE(2, 2);
    AET_MLP_CASE(2, kMlpMaxTPW);
#undef AET_MLP_CASE
}

hipError_t mlp_clear_error_flag(hipStream_t s, void *scratch, int n_clients, int B) {
    (void)B;
    unsigned long long *xrec = static_cast<unsigned long long *>(scratch);
    k_zero_words<<<1, 64, 0, s>>>(xrec + mlp_all_words(n_clients), 1);
    return hipGetLastError();
}

const int *mlp_error_flag_ptr(void *scratch, int n_clients, int B) {
    (void)B;
    unsigned long long *xrec = static_cast<unsigned long long *>(scratch);
    return reinterpret_cast<const int *>(xrec + mlp_all_words(n_clients));
}

}  // namespace aet
