// Group-sparse SwiGLU FFN over 4-bit block-quantised weights for a few tokens (2 <= T <= 16) on the
// matrix cores (paper Sec. V-A: the evaluated models are 4-bit; Sec. II-A neuron groups).
//
// Like the bf16 few-token kernels the block is bound by streaming the union of the tokens'
// surviving groups from HBM -- here a quarter of the bytes -- and the matrix instruction is a cheap
// way to apply a weight piece to all tokens at once.  With four bits per weight the operand layout
// needs no re-shaping: v_mfma_f32_16x16x32_bf16 wants, in lane l, 8 elements of row l%16 (A) and the
// same 8 elements of column l%16 (B), and WHICH 8 of a step's 32 elements lane group l/16 holds is
// free as long as A and B agree.  So lane (i, q) = (l%16, l/16) takes the 16 bytes = 32 codes
// 32q .. 32q+31 of a quantisation block of row i in one load, and step s of the block's four steps
// multiplies elements 32q + 8s .. +7 of every lane group: one load per block and lane, 64
// consecutive bytes per row, no LDS on the weight side.  A code becomes the bf16 value 128 + c with
// one and-or per pair; the block's result t = sum (128 + c) x meets the scale and the offset in float:
//     acc += s * (t - 136 * sum x)         since  s * sum (c - 8) x = s * (sum (128 + c) x - 136 sum x).
// The token side (x, or the activations) is staged in LDS with coalesced loads and read from there in
// operand order.  D: lane l holds column l%16, rows 4*(l/16)..+3.
#include "kernels.hpp"
#include "mask_device.hpp"
#include "mask_words.hpp"
#include "q4_codes.hpp"

namespace halo {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4_t mfma16q(const u32x4 &a, const u32x4 &b, const f32x4_t &c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// sum of the 8 bf16 values of a 16-byte piece
__device__ __forceinline__ float sum8(const u32x4 &v, float a)
{
    a = dot2_bf16(0x3F803F80u, v.x, a);
    a = dot2_bf16(0x3F803F80u, v.y, a);
    a = dot2_bf16(0x3F803F80u, v.z, a);
    a = dot2_bf16(0x3F803F80u, v.w, a);
    return a;
}

// ---------------------------------------------------------------------------
// gate/up.  grid: kQGateUpBlocks (+ n_pred) workgroups of 256 threads; a wave owns at most 16 of the
// union's neurons (one tile) and walks the whole row.  x is staged in LDS a range of columns at a
// time (all T tokens, up to 64 KiB); every wave multiplies its tile over that range, keeping the
// next batch of codes in flight.
// ---------------------------------------------------------------------------
constexpr int kQGateUpBlocks = 512;         // 2048 waves x 16 rows cover 256 groups
constexpr int kQBatch = 8;                  // quantisation blocks per code buffer (8 KiB per wave in flight)
constexpr int kQXBytes = 65536;             // LDS for x

struct CodeBatch {
    u32x4 v[kQBatch];                       // codes of blocks b0 .. b0+7 of row i, elements 32q..32q+31
    uint2 sc[kQBatch / 4][4];               // scales of those blocks for result rows 4q .. 4q+3
};

__global__ __launch_bounds__(256, 2) void gate_up_q4_mt(
    const bf16_t *__restrict__ x, int T, int d, int G, const uint32_t *__restrict__ Gq,
    const bf16_t *__restrict__ Gs, const uint32_t *__restrict__ Uq, const bf16_t *__restrict__ Us,
    const uint8_t *__restrict__ mask, bf16_t *__restrict__ act, int act_stride, AheadPredDev ap)
{
    constexpr int gs = 128;
    __shared__ __attribute__((aligned(16))) unsigned char s_x[kQXBytes + 16 * 16];
    __shared__ int s_list[256];
    __shared__ float s_xs[16][64];          // 136 * (sum of x[t] over quantisation block b)
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if ((int)blockIdx.x < ap.n_pred) {
        // paper Sec. III-B.3, Pred beside Load/Comp, one layer ahead: the next block's first layer
        const int j = blockIdx.x * 4 + wave;
        switch (d) {
        case 4096: predictor_row_tokens<4096>(ap.x_next, ap.At, ap.h, T, d, ap.r, j, lane); break;
        case 5120: predictor_row_tokens<5120>(ap.x_next, ap.At, ap.h, T, d, ap.r, j, lane); break;
        case 8192: predictor_row_tokens<8192>(ap.x_next, ap.At, ap.h, T, d, ap.r, j, lane); break;
        default: predictor_row_tokens<0>(ap.x_next, ap.At, ap.h, T, d, ap.r, j, lane); break;
        }
        return;
    }
    const Q4Consts qk = q4_consts();
    const MaskWords uw = load_union_words<16>(mask, T, G, lane);
    if (uw.count == 0) return;                              // nothing survives for any token (uniform): no row to read
    if (wave == 0) write_group_list(uw, lane, s_list);
    const int nblk = d / kQ4Block, words = d / 8;
    for (int idx = tid; idx < T * nblk; idx += 256) {
        const int t = idx / nblk, b = idx - t * nblk;
        const u32x4 *p = reinterpret_cast<const u32x4 *>(x + (size_t)t * d + b * kQ4Block);
        float s = 0.0f;
#pragma unroll
        for (int k = 0; k < 16; ++k) s = sum8(p[k], s);
        s_xs[t][b] = 136.0f * s;
    }
    __syncthreads();
    // this wave's tile: rows n0 .. n1-1 of the union's neurons (n1 - n0 <= 16); waves beyond the work
    // keep taking part in the barriers below with an empty tile
    // (a wave costs the same whether its tile holds 4 rows or 16, so a small union goes to fewer waves
    // with full tiles rather than to all of them)
    const long long total = (long long)uw.count * gs;
    const int waves = (gridDim.x - ap.n_pred) * 4;
    const int nw = (int)min((long long)waves, (total + 15) / 16);
    const int w = (blockIdx.x - ap.n_pred) * 4 + wave;
    const int n0 = w < nw ? (int)(total * w / nw) : 0, n1 = w < nw ? (int)(total * (w + 1) / nw) : 0;
    const int cnt = n1 - n0;
    const int i = lane & 15, q = lane >> 4;                 // operand role: row i / token i, element group q
    const int tok = i < T ? i : T - 1;                      // columns >= T repeat the last token, unused
    auto weight_row = [&](int k) -> size_t {                // tile row k -> row of the weight matrices
        const int n = cnt > 0 ? (k < cnt ? n0 + k : n1 - 1) : 0;
        const int u = n / gs;
        return (size_t)s_list[cnt > 0 ? u : 0] * gs + (n - u * gs);
    };
    const size_t arow = weight_row(i);                      // the row this lane feeds into the instruction
    size_t srow[4];                                         // the rows whose results it holds
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) srow[rr] = weight_row(4 * q + rr);
    const uint32_t *gq = Gq + arow * words + q * 4, *uq = Uq + arow * words + q * 4;
    auto fetch = [&](CodeBatch &r, const uint32_t *Q, const bf16_t *S, int b0) {
#pragma unroll
        for (int k = 0; k < kQBatch; ++k)
            r.v[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(Q + (b0 + k) * 16));
#pragma unroll
        for (int h = 0; h < kQBatch / 4; ++h)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr)
                r.sc[h][rr] = *reinterpret_cast<const uint2 *>(S + srow[rr] * nblk + b0 + 4 * h);
    };
    // x in LDS: T rows of `span` columns, pitch = span*2 + 16 bytes (16 mod 256: the 16 lanes that read
    // the same piece of different tokens hit distinct banks)
    int span = kQXBytes / (2 * T);
    span = span >= d ? d : (span / (kQBatch * kQ4Block)) * (kQBatch * kQ4Block);
    const int pitch = span * 2 + 16;
    const unsigned char *xl = s_x + tok * pitch + q * 64;   // + (block in span) * 256 + s * 16
    f32x4_t cg = {0.f, 0.f, 0.f, 0.f}, cu = {0.f, 0.f, 0.f, 0.f};
    auto multiply = [&](const CodeBatch &r, int b0, int blk_in_span, f32x4_t &acc) {
#pragma unroll
        for (int h = 0; h < kQBatch / 2; ++h) {
            // two quantisation blocks at a time: two independent chains of four matrix instructions
            f32x4_t t[2];
            u32x4 xb[2][4];
#pragma unroll
            for (int bk = 0; bk < 2; ++bk) {
                t[bk] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    xb[bk][s] = *reinterpret_cast<const u32x4 *>(xl + (blk_in_span + 2 * h + bk) * 256 + s * 16);
            }
#pragma unroll
            for (int s = 0; s < 4; ++s) {
#pragma unroll
                for (int bk = 0; bk < 2; ++bk) {
                    const u32x4 &c = r.v[2 * h + bk];
                    const uint32_t word = s == 0 ? c.x : s == 1 ? c.y : s == 2 ? c.z : c.w;
                    t[bk] = mfma16q(q4_word_bf16(word, qk), xb[bk][s], t[bk]);
                }
            }
#pragma unroll
            for (int bk = 0; bk < 2; ++bk) {
                const int blk = 2 * h + bk;                 // 0..7 within the batch: scales sc[blk / 4], element blk % 4
                const float xo = s_xs[tok][b0 + blk];
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const uint32_t pair = (blk & 2) ? r.sc[blk >> 2][rr].y : r.sc[blk >> 2][rr].x;
                    const float scale = (blk & 1) ? bf16_hi(pair) : bf16_lo(pair);
                    acc[rr] = __builtin_fmaf(scale, t[bk][rr] - xo, acc[rr]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);              // keeps one pair's operands live at a time
        }
    };
    CodeBatch R0, R1;
    const bool busy = cnt > 0;                              // a wave without rows only stages x and meets the barriers
    if (busy) fetch(R0, gq, Gs, 0);
    for (int k0 = 0; k0 < d; k0 += span) {
        const int n = min(span, d - k0);                    // columns of this range, a multiple of 1024
        __syncthreads();                                    // everybody is done with the previous range
        {
            // pieces of 16 bytes, token-major; eight loads go out before the first store (one memory
            // round trip per eight pieces and thread, not one per piece)
            const int n8 = n / 8, pieces = T * n8;
            int t = tid / n8, c = tid - t * n8;
            for (int base = tid; base < pieces; base += 256 * 8) {
                u32x4 v[8];
                int dst[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const bool ok = base + 256 * j < pieces;
                    const int tt = ok ? t : 0, cc = ok ? c : 0;
                    v[j] = *reinterpret_cast<const u32x4 *>(x + (size_t)tt * d + k0 + cc * 8);
                    dst[j] = ok ? tt * pitch + cc * 16 : -1;
                    c += 256;
                    while (c >= n8) {
                        c -= n8;
                        ++t;
                    }
                }
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (dst[j] >= 0) *reinterpret_cast<u32x4 *>(s_x + dst[j]) = v[j];
            }
        }
        __syncthreads();
        const int bfirst = k0 / kQ4Block, bend = (k0 + n) / kQ4Block;
        for (int b0 = bfirst; busy && b0 < bend; b0 += kQBatch) {
            fetch(R1, uq, Us, b0);
            multiply(R0, b0, b0 - bfirst, cg);
            fetch(R0, gq, Gs, b0 + kQBatch < nblk ? b0 + kQBatch : b0);      // past the end: a duplicate, unused
            multiply(R1, b0, b0 - bfirst, cu);
        }
    }
    // D: column = token i, rows 4q..4q+3 of the tile
    if (i < T) {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const int nn = n0 + 4 * q + rr;
            if (nn < n1) {
                const int g = s_list[nn / gs];
                const float v = mask[(size_t)i * G + g] ? silu_mul(cg[rr], cu[rr]) : 0.0f;
                act[(size_t)i * act_stride + nn] = f32_to_bf16(v);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// down.  grid: d/16 (+ n_mask) workgroups of 256 threads.  A workgroup owns 16 output rows; a group's
// 16 x 128 tile of codes is 1 KiB of consecutive bytes = one load per lane (row i, codes 32q..32q+31).
// The four waves split the union's groups, eight groups per batch: the batch's activations (T rows of
// 8 x 128 values, consecutive in the compact layout) are staged in a private LDS region with coalesced
// loads and read from there in operand order.
// ---------------------------------------------------------------------------
constexpr int kQDownGroups = 8;
constexpr int kQActPitch = kQDownGroups * 256 + 16;     // bytes per token row of a batch (16 mod 256)

// dynamic LDS of the kernel: [red: 4 x 64 x 4 floats][list: 256 ints][activations: 4 waves x T rows of
// kQActPitch bytes]; the mask workgroups use the same bytes as a MaskShared
constexpr size_t kQDownFixed = 4 * 64 * 4 * sizeof(float) + 256 * sizeof(int);
inline size_t q_down_lds_bytes(int T)
{
    const size_t need = kQDownFixed + (size_t)4 * T * kQActPitch;
    return need > sizeof(MaskShared) ? need : sizeof(MaskShared);
}

__global__ __launch_bounds__(256) void down_q4_mt(
    int T, int d, int G, const uint32_t *__restrict__ Dq, const bf16_t *__restrict__ Ds,
    const uint8_t *__restrict__ mask, const bf16_t *__restrict__ act, int act_stride, bf16_t *__restrict__ y,
    int n_mask, AheadDev nx)
{
    constexpr int gs = 128;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    if ((int)blockIdx.x < n_mask) {
        // paper Sec. III-B.3, one layer ahead: second predictor layer, ranking and mask of the next
        // block for token blockIdx.x (dispatched first: it is the longest dependent chain)
        const int t = blockIdx.x;
        mask_scores_block<256, bf16_t, true>(*reinterpret_cast<MaskShared *>(lds), threadIdx.x, nx.h + (size_t)t * nx.r,
                                             nx.Bt, nx.r, nx.scores + (size_t)t * G, G, nx.K, nx.prio_dev, nx.n_dev,
                                             nx.drop ? nx.drop + (size_t)t * nx.n_dev : nullptr,
                                             nx.order ? nx.order + (size_t)t * G : nullptr,
                                             nx.group_dev ? nx.group_dev + (size_t)t * G : nullptr,
                                             nx.mask + (size_t)t * G,
                                             nx.surv_idx ? nx.surv_idx + (size_t)t * nx.K : nullptr,
                                             nx.n_surv ? nx.n_surv + t : nullptr);
        return;
    }
    const Q4Consts qk = q4_consts();
    float(*red)[64][4] = reinterpret_cast<float(*)[64][4]>(lds);
    int *s_list = reinterpret_cast<int *>(lds + 4 * 64 * 4 * sizeof(float));
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int i = lane & 15, q = lane >> 4;
    const int j0 = (blockIdx.x - n_mask) * 16;
    const MaskWords uw = load_union_words<16>(mask, T, G, lane);
    if (wave == 0) write_group_list(uw, lane, s_list);
    __syncthreads();
    const int n_u = uw.count;
    const int u0 = n_u * wave / 4, u1 = n_u * (wave + 1) / 4;
    const int tok = i < T ? i : T - 1;
    const size_t gwords = (size_t)d * (gs / 8);                      // words per group
    const uint32_t *ctile = Dq + (size_t)(j0 + i) * (gs / 8) + q * 4;   // row i of the tile, codes 32q..32q+31
    unsigned char *mine = lds + kQDownFixed + (size_t)wave * T * kQActPitch;
    const unsigned char *al = mine + tok * kQActPitch + q * 64;      // + (group in batch) * 256 + s * 16
    f32x4_t c = {0.f, 0.f, 0.f, 0.f};
    for (int ub = u0; ub < u1; ub += kQDownGroups) {
        u32x4 r[kQDownGroups];
        uint2 sc[kQDownGroups];
#pragma unroll
        for (int k = 0; k < kQDownGroups; ++k) {
            const int u = ub + k < u1 ? ub + k : ub;                 // past the end: in-range duplicate
            const int g = s_list[u];
            r[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(ctile + g * gwords));
            sc[k] = *reinterpret_cast<const uint2 *>(Ds + (size_t)g * d + j0 + 4 * q);   // scales of rows 4q..4q+3
        }
        // the batch's activations: token t, bytes [ub*256, ub*256 + nb*256) of its row; the region is the
        // wave's own and LDS operations of a wave complete in order, so no barrier is needed
        const int nb = min(kQDownGroups, u1 - ub);
        // a token's row of the batch is 8 groups x 16 pieces; groups past the end of the wave's share
        // repeat its last one (in range, unused).  Eight loads go out before the first store.
        for (int t0 = 0; t0 < T; t0 += 4) {
            u32x4 v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int p = lane + 64 * j;                         // 0..511: token t0 + p/128, piece p%128
                const int t = min(t0 + (p >> 7), T - 1), piece = p & 127;
                const int k = min(piece >> 4, nb - 1);
                v[j] = *reinterpret_cast<const u32x4 *>(act + (size_t)t * act_stride + (size_t)(ub + k) * gs +
                                                        (piece & 15) * 8);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int p = lane + 64 * j;
                const int t = t0 + (p >> 7);
                if (t < T) *reinterpret_cast<u32x4 *>(mine + t * kQActPitch + (p & 127) * 16) = v[j];
            }
        }
#pragma unroll
        for (int k = 0; k < kQDownGroups; ++k) {
            if (k < nb) {                                            // uniform
                u32x4 b[4];
#pragma unroll
                for (int s = 0; s < 4; ++s) b[s] = *reinterpret_cast<const u32x4 *>(al + k * 256 + s * 16);
                f32x4_t t0 = {0.f, 0.f, 0.f, 0.f}, t1 = {0.f, 0.f, 0.f, 0.f};
                float asum = 0.0f;
                t0 = mfma16q(q4_word_bf16(r[k].x, qk), b[0], t0);
                t1 = mfma16q(q4_word_bf16(r[k].y, qk), b[1], t1);
                t0 = mfma16q(q4_word_bf16(r[k].z, qk), b[2], t0);
                t1 = mfma16q(q4_word_bf16(r[k].w, qk), b[3], t1);
#pragma unroll
                for (int s = 0; s < 4; ++s) asum = sum8(b[s], asum);
                const f32x4_t t = t0 + t1;
                // the four lanes of a token (one per q) hold its 128 activations between them
                asum += __shfl_xor(asum, 16);
                asum += __shfl_xor(asum, 32);
                const float xo = 136.0f * asum;
                c[0] = __builtin_fmaf(bf16_lo(sc[k].x), t[0] - xo, c[0]);
                c[1] = __builtin_fmaf(bf16_hi(sc[k].x), t[1] - xo, c[1]);
                c[2] = __builtin_fmaf(bf16_lo(sc[k].y), t[2] - xo, c[2]);
                c[3] = __builtin_fmaf(bf16_hi(sc[k].y), t[3] - xo, c[3]);
            }
        }
    }
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) red[wave][lane][rr] = c[rr];
    __syncthreads();
    if (wave == 0 && i < T) {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const float v = ((red[0][lane][rr] + red[1][lane][rr]) + red[2][lane][rr]) + red[3][lane][rr];
            y[(size_t)i * d + j0 + 4 * q + rr] = f32_to_bf16(v);
        }
    }
}

bool q4_mfma_path_supported(int T, int d, int G, int gs)
{
    return T >= 2 && T <= 16 && gs == kQ4Block && d % (kQBatch * kQ4Block) == 0 && d <= 8192 && G <= 256;
}

hipError_t launch_ffn_q4_mfma(const bf16_t *x, int T, int d, int G, const Q4Weights &w, const uint8_t *mask,
                              bf16_t *y, const DecodeScratch &ws, hipStream_t s, const AheadArgs *ahead,
                              bool *ahead_fused)
{
    const int ffn = G * kQ4Block;
    bf16_t *act = reinterpret_cast<bf16_t *>(ws.act);
    const AheadArgs *ah = (ahead && ahead_fused) ? ahead : nullptr;
    if (ahead_fused) *ahead_fused = ah != nullptr;
    const AheadPredDev ap = ahead_pred_dev(ah);
    const int n_mask = ah ? T : 0;
    const AheadDev nx = ah ? ahead_dev(*ah) : AheadDev{};
    launch_timed("gate_up_q4_mt", gate_up_q4_mt, dim3(kQGateUpBlocks + ap.n_pred), dim3(256), s, x, T, d, G, w.gate_codes,
                 w.gate_scales, w.up_codes, w.up_scales, mask, act, ffn, ap);
    static const hipError_t lds_ok = hipFuncSetAttribute(reinterpret_cast<const void *>(down_q4_mt),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize,
                                                         (int)q_down_lds_bytes(16));
    if (lds_ok != hipSuccess) return lds_ok;
    down_q4_mt<<<dim3(d / 16 + n_mask), dim3(256), q_down_lds_bytes(T), s>>>(T, d, G, w.down_codes, w.down_scales,
                                                                            mask, act, ffn, y, n_mask, nx);
    return hipGetLastError();
}

}  // namespace halo
