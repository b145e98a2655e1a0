// Group-sparse SwiGLU FFN over 4-bit block-quantised weights (paper Sec. V-A: the evaluated
// models are quantised to 4-bit integers; Sec. II-A neuron groups, merge = sum).
//
// Storage format (the library's own; the paper fixes none): blocks of 128 consecutive elements
// along the reduction dimension share one bf16 scale s, an element is s * (c - 8) with a
// 4-bit code c.  Eight codes per 32-bit word: element 2i of the eight in bits [4i, 4i+3],
// element 2i+1 in bits [16+4i, 16+4i+3], so that (word >> 4i) & 0x000F000F holds the
// pair (2i, 2i+1) in the two halves of a register -- the shape of a packed bf16 pair.
//   gate/up : codes [ffn][d/8] words, scales [ffn][d/128]        (blocks along d)
//   down    : codes [G][d][gs/8] words, scales [G][d], gs = 128  (block = the group's neurons)
//
// One token (the hot path): a quarter of the bf16 bytes per group, so the kernels are built
// like the bf16 ones -- stream every surviving byte once with 16-byte loads -- and the
// arithmetic stays far below the memory time: or-ing 0x4300 over a code gives the bf16 value
// 128 + c exactly, the packed dot instruction multiplies two of those with two activations,
// and the constant offset is taken out once per 32 elements: sum (c-8) x = sum (128+c) x -
// 136 sum x.  Any other shape goes through plain kernels that dequantise element by element.
#include "kernels.hpp"
#include "mask_device.hpp"
#include "mask_words.hpp"
#include "q4_codes.hpp"

namespace halo {

// sum over the 32 elements of one 16-byte code piece of (128 + c) * x, x as 16 packed bf16 pairs
__device__ __forceinline__ float q4_dot32(const u32x4 &c, const u32x4 (&x)[4])
{
    float a0 = 0.0f, a1 = 0.0f;
    const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        a0 = dot2_bf16(q4_pair(w[j], 0), x[j].x, a0);
        a1 = dot2_bf16(q4_pair(w[j], 1), x[j].y, a1);
        a0 = dot2_bf16(q4_pair(w[j], 2), x[j].z, a0);
        a1 = dot2_bf16(q4_pair(w[j], 3), x[j].w, a1);
    }
    return a0 + a1;
}

// sum of 32 bf16 values held as 16 packed pairs
__device__ __forceinline__ float sum32(const u32x4 (&x)[4])
{
    float a = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        a = dot2_bf16(0x3F803F80u, x[j].x, a);
        a = dot2_bf16(0x3F803F80u, x[j].y, a);
        a = dot2_bf16(0x3F803F80u, x[j].z, a);
        a = dot2_bf16(0x3F803F80u, x[j].w, a);
    }
    return a;
}

// ---------------------------------------------------------------------------
// one token, bf16 activations, d = NH * 2048, group size 128, G <= 256
// ---------------------------------------------------------------------------
// gate/up: one wave per neuron at a time, NB neurons requested together.  A lane owns the 32
// elements 2048 h + 32 lane .. + 31 of every half h: one 16-byte code piece per matrix row and
// half, one scale (block 16 h + lane / 4), and the matching 64 bytes of x kept in registers.
// Eight waves per workgroup, two per SIMD: unpacking the codes costs about three vector
// instructions per two weights, which is not negligible beside the memory time of a quarter
// of the bf16 bytes, so one wave's arithmetic has to overlap another's memory wait.
constexpr int kQ4GateUpThreads = 512;
constexpr int kQ4GateUpBlocks = 256;      // workgroups that do gate/up work (one per compute unit)

template <int NH>
__global__ __launch_bounds__(kQ4GateUpThreads, (NH == 2 ? 4 : 2)) void gate_up_q4_t1(
    const bf16_t *__restrict__ x, int G, const uint32_t *__restrict__ Gq, const bf16_t *__restrict__ Gs,
    const uint32_t *__restrict__ Uq, const bf16_t *__restrict__ Us, const uint8_t *__restrict__ mask,
    bf16_t *__restrict__ act, const bf16_t *__restrict__ x_next, const bf16_t *__restrict__ At_next, int r,
    float *__restrict__ h_next, int n_pred, int pred_rows)
{
    constexpr int d = NH * 2048, gs = 128, NB = NH == 2 ? 3 : 2, WPB = kQ4GateUpThreads / 64;
    constexpr int kWords = d / 8, kBlocks = d / kQ4Block;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    // pred_rows > 0 (then n_pred == 0): the predictor's rows are dealt evenly, pred_rows of them to the last
    // waves of every workgroup, row vblock + 256 k to wave 7 - k.  A row of At is as many bytes as two
    // neurons' codes, and a workgroup of predictor rows alone carried three quarters more bytes than its
    // neighbours' share of the codes: the compute units that held one finished 2 us after the others.
    if (pred_rows > 0 && wave >= WPB - pred_rows) {
        const int j = blockIdx.x + kQ4GateUpBlocks * (WPB - 1 - wave);
        const float p = dot_order64_fixed<d>(x_next, At_next + (size_t)j * d, lane);
        if (lane == 0) h_next[j] = p > 0.0f ? p : 0.0f;
    }
    if ((int)blockIdx.x < n_pred) {
        // the first predictor layer of the NEXT block rides along (paper Sec. III-B.3, Pred beside
        // Load/Comp, one layer ahead): one row of At per wave, h_next = ReLU(x_next A)
        const int j = blockIdx.x * WPB + wave;
        if (j < r) {
            const float p = dot_order64_fixed<d>(x_next, At_next + (size_t)j * d, lane);
            if (lane == 0) h_next[j] = p > 0.0f ? p : 0.0f;
        }
        return;
    }
    const MaskWords mw = load_mask_words(mask, G, lane);
    // contiguous runs of the surviving neurons, wave by wave (lengths differ by at most one);
    // kQ4GateUpBlocks * WPB is a power of two, and a run is far shorter than a group, so it
    // touches at most two groups: the group ids are looked up twice, not once per neuron
    constexpr int nw = kQ4GateUpBlocks * WPB;
    const int total = mw.count * gs, w = (blockIdx.x - n_pred) * WPB + wave;
    int n0 = (int)((unsigned)total * (unsigned)w / nw), n1 = (int)((unsigned)total * (unsigned)(w + 1) / nw);
    const unsigned units = (unsigned)total + 2u * (unsigned)(pred_rows * kQ4GateUpBlocks);   // a row of At = two neurons
    if (pred_rows > 0 && units >= 2u * nw) {
        // runs cut by weight: a wave that has just done a predictor row gets two neurons fewer
        auto cut = [&](int ww) {
            const int v = ww / WPB, k = ww % WPB;
            const int rows_before = v * pred_rows + (k > WPB - pred_rows ? k - (WPB - pred_rows) : 0);
            return (int)(units * (unsigned)ww / nw) - 2 * rows_before;
        };
        n0 = cut(w);
        n1 = cut(w + 1);
    }
    if (n0 >= n1) return;
    const int u_first = n0 / gs, u_last = (n1 - 1) / gs;
    const int g_first = nth_group(mw, u_first, lane), g_last = nth_group(mw, u_last, lane);
    u32x4 xr[NH][4];
    float xs[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            xr[h][j] = *reinterpret_cast<const u32x4 *>(x + h * 2048 + lane * 32 + j * 8);
    }
    for (int nb = n0; nb < n1; nb += NB) {
        u32x4 cg[NB][NH], cu[NB][NH];
        uint16_t sg[NB][NH], su[NB][NH];
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int n = nb + i < n1 ? nb + i : n1 - 1;            // past the end: an in-range duplicate
            const int u = n / gs;
            const size_t row = (size_t)(u == u_first ? g_first : g_last) * gs + (n - u * gs);
#pragma unroll
            for (int h = 0; h < NH; ++h) {
                cg[i][h] = __builtin_nontemporal_load(
                    reinterpret_cast<const u32x4 *>(Gq + row * kWords + h * 256) + lane);
                cu[i][h] = __builtin_nontemporal_load(
                    reinterpret_cast<const u32x4 *>(Uq + row * kWords + h * 256) + lane);
                sg[i][h] = Gs[row * kBlocks + h * 16 + (lane >> 2)];
                su[i][h] = Us[row * kBlocks + h * 16 + (lane >> 2)];
            }
        }
        if (nb == n0) {
#pragma unroll
            for (int h = 0; h < NH; ++h) xs[h] = 136.0f * sum32(xr[h]);
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            if (nb + i >= n1) break;                                // uniform: duplicates cost no arithmetic
            float ag = 0.0f, au = 0.0f;
#pragma unroll
            for (int h = 0; h < NH; ++h) {
                ag = __builtin_fmaf(bf16_bits_to_float(sg[i][h]), q4_dot32(cg[i][h], xr[h]) - xs[h], ag);
                au = __builtin_fmaf(bf16_bits_to_float(su[i][h]), q4_dot32(cu[i][h], xr[h]) - xs[h], au);
            }
            const float v = silu_mul_fast(wave_sum_fast(ag), wave_sum_fast(au));
            if (lane == 0) act[nb + i] = f32_to_bf16(v);
        }
    }
}

// down: four lanes share an output row j (16 bytes each = 32 of the group's 128 neurons), a
// wave covers 16 consecutive rows = 1 KiB of a group's codes, the workgroup's eight waves take
// every eighth surviving group and meet in LDS.  A lane fetches what it multiplies straight from
// memory -- its code piece, the row's scale and the 64 bytes of the activation that face the piece
// (the same 64 bytes for the 16 rows of a wave: one request per wave instruction) -- for four groups
// at a time, and takes the sum of those 32 activations itself (for the constant offset of the
// codes): nothing is staged through LDS, so no barrier stands between the mask and the first codes
// (with the activation staged once per workgroup the kernel spent 3.2 of its 5.3 us getting ready).
constexpr int kDownQ4Batch = 4;

struct DownQ4Shared {
    float part[8][16];
};

// With ahead != 0 workgroup 0 is the mask workgroup of the NEXT block (second predictor layer,
// ranking, mask); it is dispatched first because it is the longest dependent chain.  A
// workgroup is one or the other, so the two LDS layouts share their bytes and two workgroups
// fit a compute unit (the mask workgroup must run beside a down-projection one, not after).
__global__ __launch_bounds__(512, 4) void down_q4_t1(int d, int G, const uint32_t *__restrict__ Dq,
                                                      const bf16_t *__restrict__ Ds,
                                                      const uint8_t *__restrict__ mask,
                                                      const bf16_t *__restrict__ act, bf16_t *__restrict__ y,
                                                      int ahead, AheadDev nx)
{
    constexpr int gs = 128, kB = kDownQ4Batch;
    constexpr size_t kLds = sizeof(DownQ4Shared) > sizeof(MaskShared) ? sizeof(DownQ4Shared) : sizeof(MaskShared);
    __shared__ __attribute__((aligned(16))) unsigned char lds[kLds];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if (ahead && blockIdx.x == 0) {
        mask_scores_block<512, bf16_t, true>(*reinterpret_cast<MaskShared *>(lds), tid, nx.h, nx.Bt, nx.r,
                                             nx.scores, G, nx.K, nx.prio_dev, nx.n_dev, nx.drop, nx.order,
                                             nx.group_dev, nx.mask, nx.surv_idx, nx.n_surv);
        return;
    }
    DownQ4Shared &sh = *reinterpret_cast<DownQ4Shared *>(lds);
    const int vblock = blockIdx.x - (ahead ? 1 : 0);
    const MaskWords mw = load_mask_words(mask, G, lane);
    const int count = mw.count;
    const int j = vblock * 16 + (lane >> 2);                       // output row of this lane
    const int p = lane & 3;                                        // which 32 neurons of the group
    float acc = 0.0f;
    const size_t gstride = (size_t)d * 16;                         // words per group
    // this wave's groups: positions wave, wave + 8, ... of the surviving list (at most 32 of them)
    for (int u0 = wave; u0 < count; u0 += 8 * kB) {
        u32x4 c[kB], a[kB][4];
        uint16_t s[kB];
#pragma unroll
        for (int q = 0; q < kB; ++q) {
            const int u = u0 + 8 * q < count ? u0 + 8 * q : u0;      // past the end: an in-range duplicate
            const int g = nth_group(mw, u, lane);
            c[q] = __builtin_nontemporal_load(
                reinterpret_cast<const u32x4 *>(Dq + g * gstride + (size_t)j * 16) + p);
            s[q] = Ds[(size_t)g * d + j];
#pragma unroll
            for (int k = 0; k < 4; ++k) a[q][k] = *reinterpret_cast<const u32x4 *>(act + u * gs + p * 32 + k * 8);
        }
#pragma unroll
        for (int q = 0; q < kB; ++q) {
            if (u0 + 8 * q < count)
                acc = __builtin_fmaf(bf16_bits_to_float(s[q]), q4_dot32(c[q], a[q]) - 136.0f * sum32(a[q]), acc);
        }
    }
    // the four lanes of a row, then the eight waves
    acc = dpp_add<0xB1>(acc);
    acc = dpp_add<0x4E>(acc);
    if (p == 0) sh.part[wave][lane >> 2] = acc;
    __syncthreads();
    if (wave == 0 && lane < 16) {
        float v = 0.0f;
#pragma unroll
        for (int k = 0; k < 8; ++k) v += sh.part[k][lane];
        y[vblock * 16 + lane] = f32_to_bf16(v);
    }
}

// ---------------------------------------------------------------------------
// generic (any T, f32 or bf16 activations): dequantise element by element
// ---------------------------------------------------------------------------
__device__ __forceinline__ void q4_unpack8(uint32_t w, float s, float (&o)[8])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        o[2 * i] = s * (float)((int)((w >> (4 * i)) & 15u) - 8);
        o[2 * i + 1] = s * (float)((int)((w >> (16 + 4 * i)) & 15u) - 8);
    }
}

template <typename XT, int TT>
__global__ __launch_bounds__(256) void gate_up_q4_generic(
    const XT *__restrict__ x, int T, int d, int G, int gs, const uint32_t *__restrict__ Gq,
    const bf16_t *__restrict__ Gs, const uint32_t *__restrict__ Uq, const bf16_t *__restrict__ Us,
    const uint8_t *__restrict__ mask, const int32_t *__restrict__ ulist, const int32_t *__restrict__ meta,
    float *__restrict__ act, int act_stride)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int total = meta[0] * gs;
    const int nwaves = gridDim.x * 4;
    const int words = d / 8, blocks = d / kQ4Block;
    for (int n = blockIdx.x * 4 + wave; n < total; n += nwaves) {
        const int u = n / gs, m = n - u * gs;
        const int g = ulist[u];
        const size_t row = (size_t)g * gs + m;
        for (int t0 = 0; t0 < T; t0 += TT) {
            float ag[TT], au[TT];
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) ag[tt] = au[tt] = 0.0f;
            for (int c = lane; c < words; c += kWave) {
                float a[8], b[8];
                q4_unpack8(Gq[row * words + c], to_float(Gs[row * blocks + c / 16]), a);
                q4_unpack8(Uq[row * words + c], to_float(Us[row * blocks + c / 16]), b);
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) {
                    if (t0 + tt < T) {
                        float xv[8];
                        load8(x + (size_t)(t0 + tt) * d + c * 8, xv);
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            ag[tt] = __builtin_fmaf(a[e], xv[e], ag[tt]);
                            au[tt] = __builtin_fmaf(b[e], xv[e], au[tt]);
                        }
                    }
                }
            }
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                const float vg = wave_sum(ag[tt]), vu = wave_sum(au[tt]);
                const int t = t0 + tt;
                if (lane == 0 && t < T)
                    act[(size_t)t * act_stride + n] = mask[(size_t)t * G + g] ? silu_mul(vg, vu) : 0.0f;
            }
        }
    }
}

// one wave per output row j; lanes take neurons lane and lane + 64 of every union group
template <typename XT, int TT>
__global__ __launch_bounds__(256) void down_q4_generic(
    const float *__restrict__ act, int act_stride, int T, int d, const uint32_t *__restrict__ Dq,
    const bf16_t *__restrict__ Ds, const int32_t *__restrict__ ulist, const int32_t *__restrict__ meta,
    XT *__restrict__ y)
{
    constexpr int gs = 128;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int j = blockIdx.x * 4 + wave;
    if (j >= d) return;
    const int n_u = meta[0];
    for (int t0 = 0; t0 < T; t0 += TT) {
        float acc[TT];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) acc[tt] = 0.0f;
        for (int u = 0; u < n_u; ++u) {
            const size_t blk = (size_t)ulist[u] * d + j;
            const float s = to_float(Ds[blk]);
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int m = lane + half * kWave;
                const uint32_t w = Dq[blk * (gs / 8) + m / 8];
                const int k = m & 7;
                const int shift = (k & 1) ? 16 + 4 * (k >> 1) : 4 * (k >> 1);
                const float wv = s * (float)((int)((w >> shift) & 15u) - 8);
#pragma unroll
                for (int tt = 0; tt < TT; ++tt)
                    if (t0 + tt < T)
                        acc[tt] = __builtin_fmaf(wv, act[(size_t)(t0 + tt) * act_stride + u * gs + m], acc[tt]);
            }
        }
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const float v = wave_sum(acc[tt]);
            if (lane == 0 && t0 + tt < T) store_out(y + (size_t)(t0 + tt) * d + j, v);
        }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
template <typename XT>
static hipError_t q4_generic(const XT *x, int T, int d, int G, int gs, const Q4Weights &w,
                             const uint8_t *mask, XT *y, const DecodeScratch &ws, hipStream_t s)
{
    constexpr int TT = 4;
    const int ffn = G * gs;
    hipError_t e = launch_union(mask, T, G, ws.ulist, ws.meta, s);
    if (e != hipSuccess) return e;
    int blocks = (ffn + 3) / 4;
    if (blocks > 2048) blocks = 2048;
    launch_timed("gate_up_q4_generic", gate_up_q4_generic<XT, TT>, dim3(blocks), dim3(256), s, x, T, d, G, gs,
                 w.gate_codes, w.gate_scales, w.up_codes, w.up_scales, mask, (const int32_t *)ws.ulist,
                 (const int32_t *)ws.meta, ws.act, ffn);
    down_q4_generic<XT, TT><<<dim3((d + 3) / 4), dim3(256), 0, s>>>(ws.act, ffn, T, d, w.down_codes,
                                                                  w.down_scales, ws.ulist, ws.meta, y);
    return hipGetLastError();
}

bool q4_shape_supported(int d, int gs) { return gs == kQ4Block && d % kQ4Block == 0; }

bool q4_expand_supported(int T, int dtype, int d, int G, int gs)
{
    return dtype == 1 && T > 16 && q4_shape_supported(d, gs) &&
           (mfma_path_supported(T, d, gs) || prefill_path_supported(T, d, gs));
}

// 4-bit codes and their scales -> bf16 values s * (c - 8), each rounded to nearest even: rows of K elements,
// one scale per 128 consecutive elements of a row (K = d for gate / up; K = 128 with one scale per row for
// the group-blocked down projection).  A thread takes one word of codes (8 elements) at a time and writes
// 16 bytes, so that a wave's store instruction covers 1 KiB of consecutive bytes (16 bytes of codes per
// thread made every store instruction touch 64 cache lines, 16 bytes of each).
typedef float f32x2_t __attribute__((ext_vector_type(2)));

__global__ __launch_bounds__(256) void expand_q4_kernel(const uint32_t *__restrict__ codes,
                                                        const bf16_t *__restrict__ scales,
                                                        bf16_t *__restrict__ out, size_t words)
{
    constexpr int U = 4;                                    // words per thread and pass, all requested first
    const int words_per_block = kQ4Block / 8;
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t w0 = (size_t)blockIdx.x * 256 + threadIdx.x; w0 < words; w0 += stride * U) {
        uint32_t w[U];
        float s[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t i = w0 + u * stride < words ? w0 + u * stride : w0;
            w[u] = __builtin_nontemporal_load(codes + i);
            s[u] = bf16_bits_to_float(scales[i / words_per_block]);    // blocks follow each other row after row
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (w0 + u * stride < words) {
                const float off = -136.0f * s[u];
                uint32_t pr[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    // the pair (2i, 2i+1) as the bf16 values 128 + c; s * (128 + c) - 136 s = s * (c - 8), exact
                    // in float (an 8-bit by 8-bit product and a difference of neighbours); one instruction
                    // rounds both
                    const uint32_t pair = ((w[u] >> (4 * i)) & 0x000F000Fu) | 0x43004300u;
                    const f32x2_t v = {__builtin_fmaf(bf16_lo(pair), s[u], off), __builtin_fmaf(bf16_hi(pair), s[u], off)};
                    pr[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
                }
                reinterpret_cast<u32x4 *>(out)[w0 + u * stride] = u32x4{pr[0], pr[1], pr[2], pr[3]};
            }
        }
    }
}

static hipError_t expand_q4(const uint32_t *codes, const bf16_t *scales, bf16_t *out, size_t rows, int K, hipStream_t s)
{
    const size_t words = rows * (size_t)(K / 8);
    const size_t want = (words + 1023) / 1024;
    const int blocks = (int)(want < 16384 ? want : 16384);
    expand_q4_kernel<<<dim3(blocks), dim3(256), 0, s>>>(codes, scales, out, words);
    return hipGetLastError();
}

hipError_t launch_ffn_q4(int dtype, const void *x, int T, int d, int G, int gs, const Q4Weights &w,
                         const uint8_t *mask, void *y, const DecodeScratch &ws, hipStream_t s, int rank,
                         const AheadArgs *ahead, bool *ahead_fused)
{
    if (ahead_fused) *ahead_fused = false;
    if (dtype == 0)
        return q4_generic<float>((const float *)x, T, d, G, gs, w, mask, (float *)y, ws, s);
    const bf16_t *bx = (const bf16_t *)x;
    bf16_t *by = (bf16_t *)y;
    if (T == 1 && G <= 256 && (d == 4096 || d == 8192)) {
        bf16_t *act = reinterpret_cast<bf16_t *>(ws.act);
        const AheadArgs *ah = (ahead && ahead_fused) ? ahead : nullptr;
        if (ah) *ahead_fused = true;
        // predictors of 256 or 512 rows: one or two rows in every gate/up workgroup; else workgroups of their own
        const int pred_rows = (ah && (ah->r == kQ4GateUpBlocks || ah->r == 2 * kQ4GateUpBlocks)) ? ah->r / kQ4GateUpBlocks : 0;
        const int n_pred = (ah && pred_rows == 0) ? (ah->r + 7) / 8 : 0;
        const bf16_t *xn = ah ? (const bf16_t *)ah->x_next : nullptr, *an = ah ? (const bf16_t *)ah->At : nullptr;
        float *hn = ah ? ah->h : nullptr;
        const int r = ah ? ah->r : 0;
        if (d == 4096)
            launch_timed("gate_up_q4_t1", gate_up_q4_t1<2>, dim3(kQ4GateUpBlocks + n_pred), dim3(kQ4GateUpThreads), s, bx, G, w.gate_codes,
                         w.gate_scales, w.up_codes, w.up_scales, mask, act, xn, an, r, hn, n_pred, pred_rows);
        else
            launch_timed("gate_up_q4_t1", gate_up_q4_t1<4>, dim3(kQ4GateUpBlocks + n_pred), dim3(kQ4GateUpThreads), s, bx, G, w.gate_codes,
                         w.gate_scales, w.up_codes, w.up_scales, mask, act, xn, an, r, hn, n_pred, pred_rows);
        AheadDev nx{};
        if (ah) nx = ahead_dev(*ah);
        down_q4_t1<<<dim3(d / 16 + (ah ? 1 : 0)), dim3(512), 0, s>>>(d, G, w.down_codes, w.down_scales, mask, act,
                                                                     by, ah ? 1 : 0, nx);
        return hipGetLastError();
    }
    if (q4_mfma_path_supported(T, d, G, gs))
        return launch_ffn_q4_mfma(bx, T, d, G, w, mask, by, ws, s, rank, ahead, ahead_fused);
    if (ws.q4_w && q4_expand_supported(T, dtype, d, G, gs)) {
        // Many tokens and room for a block's weights as bf16: the weights are expanded once (a stream of
        // 0.5 + 2 bytes per element) and the bf16 matrix-core kernels do the rest, every weight used for
        // all the tokens that keep its group.
        const size_t ffn = (size_t)G * gs;
        bf16_t *Wg = ws.q4_w, *Wu = Wg + ffn * d, *Wd = Wu + ffn * d;
        hipError_t e = expand_q4(w.gate_codes, w.gate_scales, Wg, ffn, d, s);
        if (e == hipSuccess) e = expand_q4(w.up_codes, w.up_scales, Wu, ffn, d, s);
        if (e == hipSuccess) e = expand_q4(w.down_codes, w.down_scales, Wd, (size_t)G * d, gs, s);
        if (e != hipSuccess) return e;
        return launch_ffn_decode(dtype, x, T, d, G, gs, Wg, Wu, Wd, mask, y, ws, s);
    }
    if (T > 16 && q4_mfma_path_supported(16, d, G, gs)) {
        // Many tokens: the matrix-core kernels over tiles of up to 16 tokens, one tile after the other on
        // the stream (each streams the union of its own tokens' groups; the activation scratch is reused).
        // No kernel of its own for this case yet: a tile pair of launches is 30-90 us, where the plain path
        // below takes 50 us per TOKEN at the 7B shape.  A last tile of one token would leave the kernels'
        // range, so the last two tiles share their tokens.
        for (int t0 = 0; t0 < T;) {
            int n = T - t0 > 16 ? 16 : T - t0;
            if (T - t0 == 17) n = 15;
            const hipError_t e = launch_ffn_q4_mfma(bx + (size_t)t0 * d, n, d, G, w, mask + (size_t)t0 * G,
                                                    by + (size_t)t0 * d, ws, s, rank, nullptr, nullptr);
            if (e != hipSuccess) return e;
            t0 += n;
        }
        return hipSuccess;
    }
    return q4_generic<bf16_t>(bx, T, d, G, gs, w, mask, by, ws, s);
}

}  // namespace halo
