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
// consecutive bytes per row, no LDS on the weight side.  (The gate/up kernel fetches the same bytes
// whole cache lines at a time, two blocks of eight rows per instruction, and gets to this layout with
// lane-crossing moves: see CodeBatch.)  A code becomes the bf16 value 128 + c with
// one and-or per pair; the block's result t = sum (128 + c) x meets the scale and the offset in float:
//     acc += s * (t - 136 * sum x)         since  s * sum (c - 8) x = s * (sum (128 + c) x - 136 sum x).
// The token side (x, or the activations) is staged in LDS with coalesced loads and read from there in
// operand order.  D: lane l holds column l%16, rows 4*(l/16)..+3.
#include <type_traits>

#include "kernels.hpp"
#include "mask_device.hpp"
#include "mask_words.hpp"
#include "q4_codes.hpp"

namespace halo {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// From the loaded layout (a: tile rows r, b: rows 8 + r; lanes with bit 3 clear hold the pair's first
// block, lanes with bit 3 set its second) to the operand layout (lane = 16q + row): c0 = first block, c1 =
// second block of the pair.  Row i < 8 of c0 is a's own lane, row 8 + r is b's lane across bit 3; c1 the
// other way round.  Crossing bit 3 is a rotation by 8 within a row of 16 lanes (DPP row_ror:8); the bank
// mask writes lanes 8..15 (0xC) or 0..7 (0x3) and leaves the others as they were.
__device__ __forceinline__ uint32_t cross8(uint32_t keep, uint32_t take, int banks_hi)
{
    return banks_hi ? (uint32_t)__builtin_amdgcn_update_dpp((int)keep, (int)take, 0x128, 0xf, 0xC, false)
                    : (uint32_t)__builtin_amdgcn_update_dpp((int)keep, (int)take, 0x128, 0xf, 0x3, false);
}
__device__ __forceinline__ void operand_pair(const u32x4 &a, const u32x4 &b, u32x4 &c0, u32x4 &c1)
{
    c0 = u32x4{cross8(a.x, b.x, 1), cross8(a.y, b.y, 1), cross8(a.z, b.z, 1), cross8(a.w, b.w, 1)};
    c1 = u32x4{cross8(b.x, a.x, 0), cross8(b.y, a.y, 0), cross8(b.z, a.z, 0), cross8(b.w, a.w, 0)};
}

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
// gate/up.  grid: one workgroup of eight waves, or two of four, per compute unit; every workgroup does the
// same kind of work.  The union's neurons are cut into tiles of up to 16 rows and a workgroup owns a run
// of consecutive tiles.  Its work is the run's (tile, pair of quantisation blocks) items in row-major
// order, and its waves take equal runs of THOSE: a wave multiplies a stretch of the reduction range of at
// most three tiles, keeps the partial sums in registers, and the partial sums of a tile meet in LDS once,
// when all of the workgroup's streaming is done.  (A wave per tile walking the whole row left three
// quarters of the waves idle on a 63-group union and all the work on a quarter of the compute units; a
// reduction per tile cost two barriers and a row set-up per 3 us of multiplying.)
// A wave always has one batch of gate codes and one of up codes in flight; x (all T tokens) is staged in
// LDS, whole, or in two halves of the row when it is larger than the LDS.
// The first predictor layer of the next block (paper Sec. III-B.3, Pred beside Load/Comp, one layer
// ahead) is dealt over the same workgroups, a row of At to a wave, after the wave's stretch; such a wave
// gets a shorter stretch, by the pairs of blocks a row costs.  Workgroups of predictor rows alone would
// each hold a compute unit's slot (the LDS for x) while doing none of the streaming.
// ---------------------------------------------------------------------------
constexpr int kQBatch = 8;                  // quantisation blocks per code buffer (8 KiB per wave in flight)
// LDS for x: 64 KiB in a workgroup of four waves, two to a compute unit; when the T tokens' rows need more,
// 128 KiB in a workgroup of eight waves, one to a compute unit.  Either way eight waves share the unit.
constexpr int q_x_bytes(int waves) { return waves == 4 ? 65536 : 131072; }
constexpr int q_gate_up_blocks(int waves) { return 2048 / waves; }

// Codes as they are loaded: one instruction covers whole 128-byte lines -- a pair of blocks of eight rows --
// because a load of 64 bytes of each of 16 rows (the operand layout itself) asks the cache for twice the
// lines and streamed a third slower.  Lane l = (q, bk, r) = (l / 16, l / 8 % 2, l % 8): v[2p] holds 16 bytes
// of tile row r, v[2p + 1] of tile row 8 + r, both the codes 32q..32q+31 of block 2p + bk of the batch.
// operand_pair() turns the two into the operand layout with four lane-crossing moves each.
struct CodeBatch {
    u32x4 v[kQBatch];
    uint32_t sc[kQBatch / 2][4];            // scales of block pairs (b0+2p, b0+2p+1) for result rows 4q .. 4q+3
};

// where a lane's operand row and its four result rows of a tile start
struct QTile {
    int aoff[2];                            // word offsets of (tile row r, 8 + r; this lane's 16 bytes of a pair of blocks)
    int soff[4];                            // element offsets of the result rows in a scale matrix
};

template <int WAVES>
__global__ __launch_bounds__(WAVES * 64, 8 / WAVES) void gate_up_q4_mt(
    const bf16_t *__restrict__ x, int T, int d, int G, const uint32_t *__restrict__ Gq,
    const bf16_t *__restrict__ Gs, const uint32_t *__restrict__ Uq, const bf16_t *__restrict__ Us,
    const uint8_t *__restrict__ mask, bf16_t *__restrict__ act, int act_stride, AheadPredDev ap)
{
    constexpr int gs = 128;
    constexpr int kQXBytes = q_x_bytes(WAVES);
    // x; at the very end the same bytes hold the waves' partial sums, [tile][wave][lane][gate 0..3, up 4..7]
    __shared__ __attribute__((aligned(16))) unsigned char s_x[kQXBytes + 16 * 16];
    __shared__ int s_list[256];
    __shared__ float s_xs[16][64];          // 136 * (sum of x[t] over quantisation block b)
    static_assert(WAVES * WAVES * 64 * 8 * sizeof(float) <= kQXBytes, "partial sums of a workgroup's tiles fit");
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // in a scalar register: what depends on it is uniform
    const Q4Consts qk = q4_consts();
    const int i = lane & 15, q = lane >> 4;                 // operand role: row i / token i, element group q
    const int tok = i < T ? i : T - 1;                      // columns >= T repeat the last token, unused
    // x in LDS: T rows of `span` columns (the row, or half of it), pitch = span*2 + 16 bytes (16 mod 256:
    // the 16 lanes that read the same piece of different tokens hit distinct banks)
    const int nspans = (T * d * 2 + kQXBytes - 1) / kQXBytes;      // 1 or 2, by the host's choice of WAVES
    const int span = d / nspans, bps = span / kQ4Block, ppr = bps / 2;
    const int pitch = span * 2 + 16;
    const unsigned char *xl = s_x + tok * pitch + q * 64;   // + (block in span) * 256 + s * 16
    // Columns k0 .. k0+span-1 of all tokens go straight to LDS, 1 KiB (512 columns of one token) per wave
    // and instruction, no registers in between: the requests are out before the mask bytes are asked for,
    // and the weight rows requested once the union is known travel beside them.
    const uint32_t s_x_addr = (uint32_t)(size_t)s_x;
    auto x_request = [&](int k0) {
        const int cpr = span / 512, chunks = T * cpr;       // chunks of a token row, chunks in all: <= kQXBytes / 1024
        for (int c = wave; c < chunks; c += WAVES) {        // uniform
            const int t = c / cpr, part = c - t * cpr;
            load_to_lds16_all(x, (uint32_t)(t * d + k0 + part * 512 + lane * 8) * 2u, s_x_addr + t * pitch + part * 1024);
        }
    };
    // 136 * the sum of every (token, quantisation block) of the range: a wave sums the chunks it asked for
    // itself (after its own wait for them, no barrier in between); a chunk is four blocks, 16 lanes a block
    auto x_sums = [&](int k0) {
        const int cpr = span / 512, chunks = T * cpr;
        for (int c = wave; c < chunks; c += WAVES) {        // uniform
            const int t = c / cpr, part = c - t * cpr;
            float sum = sum8(*reinterpret_cast<const u32x4 *>(s_x + t * pitch + part * 1024 + lane * 16), 0.0f);
            sum = xor_add<8>(sum);
            sum = xor_add<4>(sum);
            sum = xor_add<2>(sum);
            sum = xor_add<1>(sum);
            if ((lane & 15) == 0) s_xs[t][k0 / kQ4Block + part * 4 + (lane >> 4)] = 136.0f * sum;
        }
    };
    x_request(0);
    // the union of the tokens' surviving groups, eight tokens' mask bytes per memory round trip
    MaskWords uw;
    {
        uint32_t any[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int t0 = 0; t0 < 16; t0 += 8) {
            if (t0 < T) {                                   // uniform
                uint8_t v[8][4];
#pragma unroll
                for (int t = 0; t < 8; ++t)
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const int g = k * kWave + lane;
                        v[t][k] = mask[(uint32_t)((t0 + t < T ? t0 + t : T - 1) * G + (g < G ? g : 0))];
                    }
#pragma unroll
                for (int t = 0; t < 8; ++t)
#pragma unroll
                    for (int k = 0; k < 4; ++k) any[k] |= v[t][k];
            }
        }
        uw.count = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            uw.w[k] = __ballot(k * kWave + lane < G && any[k] != 0u);
            uw.count += __popcll(uw.w[k]);
        }
    }
    const int total = uw.count * gs;
    const int nt = (total + 15) / 16;                       // tiles; rows dealt evenly, at most 16 each
    const int rows_lo = nt ? total / nt : 0, rows_rem = nt ? total - rows_lo * nt : 0;
    auto tile_begin = [&](int t) { return t * rows_lo + min(t, rows_rem); };
    const int nwg = gridDim.x, wg = blockIdx.x;
    const int t_lo = nt * wg / nwg, ntw = nt * (wg + 1) / nwg - t_lo;           // this workgroup's tiles: <= WAVES
    // predictor rows of this workgroup; without an overlapped next step (n_pred == 0) they are not computed, but the
    // waves' stretches are cut as if they were, so that a block's output has the same bits either way
    const int j_lo = (int)((long long)ap.r * wg / nwg), npr = (int)((long long)ap.r * (wg + 1) / nwg) - j_lo;
    const int npr_run = ap.n_pred ? npr : 0;
    if (ntw == 0 && npr_run == 0) return;                   // uniform
    // predictor rows go to the last waves first: row j_lo + k to wave WAVES-1 - k % WAVES
    auto rows_of_wave = [&](int v) { const int k0 = WAVES - 1 - v; return k0 < npr ? (npr - k0 + WAVES - 1) / WAVES : 0; };
    // the cut of the workgroup's ntw * ppr pairs of blocks between the waves; `weight` = pairs a predictor row counts for
    const int P = ntw * ppr;
    int cut[WAVES + 1] = {};
    auto make_cuts = [&](int weight) {
        const int U = P + weight * npr;
        int rows_before = 0, worst = 0;
        cut[0] = 0;
#pragma unroll
        for (int v = 0; v < WAVES; ++v) {
            rows_before += rows_of_wave(v);
            int c = v == WAVES - 1 ? P : U * (v + 1) / WAVES - weight * rows_before;
            c = c < cut[v] ? cut[v] : c > P ? P : c;
            cut[v + 1] = c;
            if (c > cut[v]) worst = max(worst, (c - 1) / ppr - cut[v] / ppr + 1);
        }
        return worst;                                       // the most tiles any wave's stretch touches
    };
    if (ntw > 0) {
        // a row of At for T tokens is about T * d / 512 * 24 vector instructions, a pair of blocks of gate and
        // up about 250; the stretches must stay within three tiles (three sets of partial sums per wave)
        int weight = T * (d / 512) / 10;
        weight = weight < 1 ? 1 : weight > ppr ? ppr : weight;
        if (make_cuts(npr ? weight : 0) > 3) make_cuts(0);
    }
    int p0 = 0, p1 = 0;                                     // (selected, not indexed: the cuts stay in registers)
    if (ntw > 0) {
#pragma unroll
        for (int v = 0; v < WAVES; ++v)
            if (v == wave) {
                p0 = cut[v];
                p1 = cut[v + 1];
            }
    }
    const int tl0 = ntw > 0 ? p0 / ppr : 0, npieces = p1 > p0 ? (p1 - 1) / ppr - tl0 + 1 : 0;
    const int nblk = d / kQ4Block, words = d / 8;
    // the tile this wave finishes at the end (local index = wave): whether token i keeps its groups
    uint8_t keep_first = 0, keep_last = 0;
    int fin_n0 = 0, fin_n1 = 0;
    if (ntw > 0) {
        if (wave == 0) write_group_list(uw, lane, s_list);
        __syncthreads();                                    // the list
        if (wave < ntw) {
            fin_n0 = tile_begin(t_lo + wave);
            fin_n1 = tile_begin(t_lo + wave + 1);
            keep_first = mask[(size_t)tok * G + s_list[fin_n0 / gs]];
            keep_last = mask[(size_t)tok * G + s_list[(fin_n1 - 1) / gs]];
        }
    }
    auto setup = [&](QTile &t, int tile) {
        const int n0 = tile_begin(tile), n1 = tile_begin(tile + 1);
        auto weight_row = [&](int k) -> int {               // tile row k -> row of the weight matrices
            const int n = n0 + k < n1 ? n0 + k : n1 - 1;
            const int u = n / gs;
            return s_list[u] * gs + (n - u * gs);
        };
        const int bk = (lane >> 3) & 1;
        t.aoff[0] = weight_row(lane & 7) * words + bk * 16 + q * 4;
        t.aoff[1] = weight_row(8 + (lane & 7)) * words + bk * 16 + q * 4;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) t.soff[rr] = weight_row(4 * q + rr) * nblk;
    };
    // piece k of this wave's stretch within the range of columns rg: blocks [b_lo, b_hi) of tile tl0 + k
    auto piece_blocks = [&](int rg, int k, int &b_lo, int &b_hi) {
        const int first = (tl0 + k) * ppr;
        b_lo = rg * bps + 2 * (max(p0, first) - first);
        b_hi = rg * bps + 2 * (min(p1, first + ppr) - first);
    };
    // blocks b0 .. b0+7 of the lane's rows, as far as they lie below `end` (uniform conditions)
    auto fetch = [&](CodeBatch &r_, const uint32_t *Q, const bf16_t *S, const QTile &t, int b0, int end) {
#pragma unroll
        for (int k = 0; k < kQBatch; ++k)
            if (b0 + (k & ~1) < end)
                r_.v[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(Q + t.aoff[k & 1] + (b0 + (k & ~1)) * 16));
#pragma unroll
        for (int h = 0; h < kQBatch / 2; ++h)
            if (b0 + 2 * h < end) {
#pragma unroll
                for (int rr = 0; rr < 4; ++rr)
                    r_.sc[h][rr] = *reinterpret_cast<const uint32_t *>(S + t.soff[rr] + b0 + 2 * h);
            }
    };
    // Multiplies blocks b0 .. of the buffer (below `end`); as soon as a pair of blocks has been used, its
    // registers are asked for the same pair of the buffer's next batch (blocks n0 .. below nend of the rows of
    // nt_), so a wave's two buffers stay in flight all the time instead of one being idle while it is used.
    auto multiply = [&](CodeBatch &r_, int b0, int end, int bfirst, f32x4_t &acc, const uint32_t *Q, const bf16_t *S,
                        const QTile &nt_, int n0, int nend) {
#pragma unroll
        for (int h = 0; h < kQBatch / 2; ++h) {
            if (b0 + 2 * h >= end && n0 + 2 * h >= nend) break;         // uniform
            if (b0 + 2 * h < end) {
            // two quantisation blocks at a time: two independent chains of four matrix instructions
            f32x4_t t[2];
            u32x4 xb[2][4], c[2];
            operand_pair(r_.v[2 * h], r_.v[2 * h + 1], c[0], c[1]);
#pragma unroll
            for (int bk = 0; bk < 2; ++bk) {
                t[bk] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    xb[bk][s] = *reinterpret_cast<const u32x4 *>(xl + (b0 - bfirst + 2 * h + bk) * 256 + s * 16);
            }
#pragma unroll
            for (int s = 0; s < 4; ++s) {
#pragma unroll
                for (int bk = 0; bk < 2; ++bk) {
                    const uint32_t word = s == 0 ? c[bk].x : s == 1 ? c[bk].y : s == 2 ? c[bk].z : c[bk].w;
                    t[bk] = mfma16q(q4_word_bf16(word, qk), xb[bk][s], t[bk]);
                }
            }
#pragma unroll
            for (int bk = 0; bk < 2; ++bk) {
                const float xo = s_xs[tok][b0 + 2 * h + bk];
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const float scale = bk ? bf16_hi(r_.sc[h][rr]) : bf16_lo(r_.sc[h][rr]);
                    acc[rr] = __builtin_fmaf(scale, t[bk][rr] - xo, acc[rr]);
                }
            }
            }
            if (n0 + 2 * h < nend) {                        // uniform
                r_.v[2 * h] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(Q + nt_.aoff[0] + (n0 + 2 * h) * 16));
                r_.v[2 * h + 1] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(Q + nt_.aoff[1] + (n0 + 2 * h) * 16));
#pragma unroll
                for (int rr = 0; rr < 4; ++rr)
                    r_.sc[h][rr] = *reinterpret_cast<const uint32_t *>(S + nt_.soff[rr] + n0 + 2 * h);
            }
            __builtin_amdgcn_sched_barrier(0);              // keeps one pair's operands live at a time
        }
    };
    // partial sums of the (up to three) tiles of the stretch
    f32x4_t sg[3], su[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) sg[k] = su[k] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    if (ntw > 0) {
        QTile cur;
        CodeBatch R0, R1;                                   // gate and up codes of the same blocks
        for (int rg = 0; rg < nspans; ++rg) {               // uniform
            if (rg > 0) {
                __syncthreads();                            // everybody is done with the previous range
                x_request(rg * span);
            }
            int wb0 = 0, wb1 = 0;
            if (npieces > 0) {
                setup(cur, t_lo + tl0);
                piece_blocks(rg, 0, wb0, wb1);
                fetch(R0, Gq, Gs, cur, wb0, wb1);
                fetch(R1, Uq, Us, cur, wb0, wb1);
            }
            wait_all_loads();                               // x is in LDS (and the first batches are here)
            x_sums(rg * span);
            __syncthreads();
            for (int k = 0; k < npieces; ++k) {
                f32x4_t cg = k == 0 ? sg[0] : k == 1 ? sg[1] : sg[2];
                f32x4_t cu = k == 0 ? su[0] : k == 1 ? su[1] : su[2];
                int nb0 = 0, nb1 = 0;                       // the next piece of this range, if any
                if (k + 1 < npieces) piece_blocks(rg, k + 1, nb0, nb1);
                for (int b0 = wb0; b0 < wb1; b0 += kQBatch) {
                    // the buffers are refilled from the same rows, or, in the piece's last batch, from the
                    // next piece's rows if there is one
                    const bool last = b0 + kQBatch >= wb1;
                    if (last && k + 1 < npieces) setup(cur, t_lo + tl0 + k + 1);
                    const int rn0 = last ? nb0 : b0 + kQBatch, rn1 = last ? nb1 : wb1;
                    multiply(R0, b0, wb1, rg * bps, cg, Gq, Gs, cur, rn0, rn1);
                    multiply(R1, b0, wb1, rg * bps, cu, Uq, Us, cur, rn0, rn1);
                }
                if (k == 0) {
                    sg[0] = cg;
                    su[0] = cu;
                } else if (k == 1) {
                    sg[1] = cg;
                    su[1] = cu;
                } else {
                    sg[2] = cg;
                    su[2] = cu;
                }
                wb0 = nb0;
                wb1 = nb1;
            }
        }
    }
    // this wave's predictor rows
    for (int k = WAVES - 1 - wave; k < npr_run; k += WAVES) {
        const int j = j_lo + k;
        switch (d) {
        case 4096: predictor_row_tokens_batched<4096, 2>(ap.x_next, ap.At, ap.h, T, ap.r, j, lane); break;
        case 5120: predictor_row_tokens_batched<5120, 2>(ap.x_next, ap.At, ap.h, T, ap.r, j, lane); break;
        case 8192: predictor_row_tokens<8192>(ap.x_next, ap.At, ap.h, T, d, ap.r, j, lane); break;
        default: predictor_row_tokens<0>(ap.x_next, ap.At, ap.h, T, d, ap.r, j, lane); break;
        }
    }
    if (ntw == 0) return;                                   // uniform
    __syncthreads();                                        // nobody reads x any more: its bytes take the partial sums
    float *part = reinterpret_cast<float *>(s_x);
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        if (k < npieces) {
            float *dst = part + ((size_t)((tl0 + k) * WAVES + wave) * 64 + lane) * 8;
            *reinterpret_cast<f32x4_t *>(dst) = sg[k];
            *reinterpret_cast<f32x4_t *>(dst + 4) = su[k];
        }
    }
    __syncthreads();
    // wave v finishes tile v of the workgroup: the stretches that touch it, in the order of the row.
    // D: column = token i, rows 4q..4q+3 of the tile
    if (wave < ntw) {
        f32x4_t g_ = {0.f, 0.f, 0.f, 0.f}, u_ = {0.f, 0.f, 0.f, 0.f};
        const int first = wave * ppr;
#pragma unroll
        for (int v = 0; v < WAVES; ++v) {
            if (cut[v] < first + ppr && cut[v + 1] > first && cut[v + 1] > cut[v]) {        // uniform
                const float *src = part + ((size_t)(wave * WAVES + v) * 64 + lane) * 8;
                const f32x4_t a = *reinterpret_cast<const f32x4_t *>(src), b = *reinterpret_cast<const f32x4_t *>(src + 4);
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    g_[rr] += a[rr];
                    u_[rr] += b[rr];
                }
            }
        }
        if (i < T) {
            const int u_first = fin_n0 / gs;
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int nn = fin_n0 + 4 * q + rr;
                if (nn < fin_n1) {
                    const uint8_t keep = nn / gs == u_first ? keep_first : keep_last;
                    act[(size_t)i * act_stride + nn] = f32_to_bf16(keep ? silu_mul(g_[rr], u_[rr]) : 0.0f);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// down.  A workgroup owns 16 * TILES output rows; a group's 16 x 128 tile of codes is 1 KiB of consecutive
// bytes = one load per lane (row i, codes 32q..32q+31).  The waves split the union's groups, GB groups per
// batch.  The codes and scales of a group are asked for again, for the next batch, as soon as they have been
// used; the next batch's activations (T rows of GB x 128 values, consecutive in the compact layout) are
// requested into registers before the current batch is multiplied and written to the wave's private LDS
// region, from where they are read in operand order, once the multiplication is done with the region.
// (With one batch at a time -- loads, wait, activations, wait, multiply -- a wave waited for memory three
// times per eight groups and the kernel ran at 1.5 TB/s.)
// Every workgroup reads all of the tokens' activations, T * 256 bytes per group beside the 1 KiB of codes
// of a 16-row tile: with eight tokens that is twice the codes' bytes, and the loads a compute unit can
// have in flight are what bounds the kernel.  TILES = 2 (eight waves, 32 rows: long rows, d >= 8192, where
// d/32 workgroups still cover the chip) uses every activation byte for two tiles.
// TMAX: the token rows a wave fetches per batch (rows past T repeat the last token's, unused): fixed at
// compile time so that every load is issued unconditionally and the compiler can count the loads in flight.
// grid: d / (16 * TILES) (+ n_mask) workgroups of 64 * WAVES threads.
// ---------------------------------------------------------------------------
// dynamic LDS of the kernel: [list: 256 ints][activations: WAVES x T rows of GB * 256 + 16 bytes (16 mod 256)];
// at the end a wave's partial sums (64 x 4 TILES floats <= 2 rows) take the place of its activations; the mask
// workgroups use the same bytes as a MaskShared
constexpr size_t kQDownFixed = 256 * sizeof(int);
constexpr int q_act_pitch(int gb) { return gb * 256 + 16; }
// a wave's region: its T activation rows, and room for its partial sums
__host__ __device__ inline size_t q_down_region(int T, int gb, int tiles)
{
    const size_t rows = (size_t)T * q_act_pitch(gb), sums = (size_t)64 * 4 * tiles * sizeof(float);
    return rows > sums ? rows : sums;
}
inline size_t q_down_lds_bytes(int T, int waves, int gb, int tiles)
{
    const size_t need = kQDownFixed + (size_t)waves * q_down_region(T, gb, tiles);
    return need > sizeof(MaskShared) ? need : sizeof(MaskShared);
}

template <int TILES, int GB>
struct DownBatch {
    u32x4 r[TILES][GB];                     // codes of the batch's groups: row i of each tile, codes 32q..32q+31
    uint2 sc[TILES][GB];                    // scales of rows 4q .. 4q+3 of each tile
};

// GB: groups per batch (4; 2 in the 32-row form, whose registers then leave room for two workgroups of
// eight waves on a compute unit: with one, the mask workgroups in front of the grid held eight units for
// themselves and as many projection workgroups started when they were done).
template <int TMAX, int TILES, int WAVES, int GB>
__global__ __launch_bounds__(WAVES * 64) void down_q4_mt(
    int T, int d, int G, const uint32_t *__restrict__ Dq, const bf16_t *__restrict__ Ds,
    const uint8_t *__restrict__ mask, const bf16_t *__restrict__ act, int act_stride, bf16_t *__restrict__ y,
    int n_mask, AheadDev nx)
{
    constexpr int gs = 128, kPitch = q_act_pitch(GB);
    constexpr int kLanesPerToken = GB * 16, kTokPerLoad = 64 / kLanesPerToken, kActLoads = (TMAX + kTokPerLoad - 1) / kTokPerLoad;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    if ((int)blockIdx.x < n_mask) {
        // paper Sec. III-B.3, one layer ahead: second predictor layer, ranking and mask of the next
        // block for token blockIdx.x (dispatched first: it is the longest dependent chain)
        const int t = blockIdx.x;
        mask_scores_block<WAVES * 64, bf16_t, true>(
            *reinterpret_cast<MaskShared *>(lds), threadIdx.x, nx.h + (size_t)t * nx.r, nx.Bt, nx.r,
            nx.scores + (size_t)t * G, G, nx.K, nx.prio_dev, nx.n_dev, nx.drop ? nx.drop + (size_t)t * nx.n_dev : nullptr,
            nx.order ? nx.order + (size_t)t * G : nullptr, nx.group_dev ? nx.group_dev + (size_t)t * G : nullptr,
            nx.mask + (size_t)t * G, nx.surv_idx ? nx.surv_idx + (size_t)t * nx.K : nullptr,
            nx.n_surv ? nx.n_surv + t : nullptr);
        return;
    }
    const Q4Consts qk = q4_consts();
    int *s_list = reinterpret_cast<int *>(lds);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i = lane & 15, q = lane >> 4;
    const int j0 = (blockIdx.x - n_mask) * 16 * TILES;
    const MaskWords uw = load_union_words<16>(mask, T, G, lane);
    if (wave == 0) write_group_list(uw, lane, s_list);
    __syncthreads();
    const int n_u = uw.count;
    const int u0 = n_u * wave / WAVES, u1 = n_u * (wave + 1) / WAVES;
    const int nbat = (u1 - u0 + GB - 1) / GB;
    const int tok = i < T ? i : T - 1;
    const size_t gwords = (size_t)d * (gs / 8);                      // words per group
    const uint32_t *ctile = Dq + (size_t)(j0 + i) * (gs / 8) + q * 4;   // row i of the first tile, codes 32q..32q+31
    const size_t region = q_down_region(T, GB, TILES);
    unsigned char *mine = lds + kQDownFixed + (size_t)wave * region;
    const unsigned char *al = mine + tok * kPitch + q * 64;          // + (group in batch) * 256 + s * 16
    f32x4_t c[TILES];
#pragma unroll
    for (int tl = 0; tl < TILES; ++tl) c[tl] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    // the wave's groups (at most 64: G <= 256 over at least four waves), one to a lane: a batch's group ids
    // come out of this register into scalar registers, where reading the list from LDS put a dependent LDS
    // round trip and vector address arithmetic in front of every batch's loads (0.6 us per batch of four)
    const int my_group = s_list[min(u0 + lane, max(u1 - 1, 0))];
    // Batch b of the wave's share is groups u0 + GB b ..; those past the end of the share repeat its last one
    // (in range, unused).  Codes and scales of group k of a batch:
    DownBatch<TILES, GB> B;
    auto load_group = [&](int b, int k) {
        const int g = __builtin_amdgcn_readlane(my_group, min(u0 + b * GB + k, u1 - 1) - u0);
#pragma unroll
        for (int tl = 0; tl < TILES; ++tl) {
            B.r[tl][k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(ctile + g * gwords + tl * 16 * (gs / 8)));
            B.sc[tl][k] = *reinterpret_cast<const uint2 *>(Ds + (size_t)g * d + j0 + 16 * tl + 4 * q);   // rows 4q..4q+3
        }
    };
    // A token's row of a batch is GB groups x 16 pieces of 16 bytes: one piece per lane, 4 / GB tokens per load.
    u32x4 av[kActLoads];
    const int a_tok = lane / kLanesPerToken, a_piece = lane % kLanesPerToken;
    auto load_act = [&](int b) {
        const int un = min(u0 + b * GB + (a_piece >> 4), u1 - 1);    // position in the union of this lane's piece
#pragma unroll
        for (int j = 0; j < kActLoads; ++j)
            av[j] = *reinterpret_cast<const u32x4 *>(act + (size_t)min(j * kTokPerLoad + a_tok, T - 1) * act_stride +
                                                     (size_t)un * gs + (a_piece & 15) * 8);
    };
    // the region is the wave's own and LDS operations of a wave complete in order, so no barrier is needed
    auto store_act = [&]() {
#pragma unroll
        for (int j = 0; j < kActLoads; ++j) {
            const int t = j * kTokPerLoad + a_tok;
            if (t < T) *reinterpret_cast<u32x4 *>(mine + t * kPitch + a_piece * 16) = av[j];
        }
    };
    // Multiplies the first nb groups of the batch in B.  `refill`: as soon as a group's registers are used
    // they are asked for the same group of batch b + 1 (a full batch: no condition, so the compiler can count
    // the loads in flight), and the batch is whole.
    auto multiply = [&](auto refill, int b, int nb) {
        constexpr bool kRefill = decltype(refill)::value;
#pragma unroll
        for (int k = 0; k < GB; ++k) {
            if (kRefill || k < nb) {                                 // uniform
                u32x4 xb[4];
#pragma unroll
                for (int s = 0; s < 4; ++s) xb[s] = *reinterpret_cast<const u32x4 *>(al + k * 256 + s * 16);
                // the sum of the token's 128 activations of the group, for the offset: the same matrix
                // instructions with 1.0 in every element of the other operand (every row of the result is the
                // sum).  Summing the lane's 32 values and exchanging between the token's four lanes was a
                // chain of two lane-crossing round trips per group, in a loop that has nothing to hide them.
                const u32x4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
                f32x4_t ts0 = {0.f, 0.f, 0.f, 0.f}, ts1 = {0.f, 0.f, 0.f, 0.f};
                ts0 = mfma16q(ones, xb[0], ts0);
                ts1 = mfma16q(ones, xb[1], ts1);
                ts0 = mfma16q(ones, xb[2], ts0);
                ts1 = mfma16q(ones, xb[3], ts1);
                const float xo = 136.0f * (ts0[0] + ts1[0]);
#pragma unroll
                for (int tl = 0; tl < TILES; ++tl) {
                    f32x4_t t0 = {0.f, 0.f, 0.f, 0.f}, t1 = {0.f, 0.f, 0.f, 0.f};
                    t0 = mfma16q(q4_word_bf16(B.r[tl][k].x, qk), xb[0], t0);
                    t1 = mfma16q(q4_word_bf16(B.r[tl][k].y, qk), xb[1], t1);
                    t0 = mfma16q(q4_word_bf16(B.r[tl][k].z, qk), xb[2], t0);
                    t1 = mfma16q(q4_word_bf16(B.r[tl][k].w, qk), xb[3], t1);
                    const f32x4_t t = t0 + t1;
                    c[tl][0] = __builtin_fmaf(bf16_lo(B.sc[tl][k].x), t[0] - xo, c[tl][0]);
                    c[tl][1] = __builtin_fmaf(bf16_hi(B.sc[tl][k].x), t[1] - xo, c[tl][1]);
                    c[tl][2] = __builtin_fmaf(bf16_lo(B.sc[tl][k].y), t[2] - xo, c[tl][2]);
                    c[tl][3] = __builtin_fmaf(bf16_hi(B.sc[tl][k].y), t[3] - xo, c[tl][3]);
                }
                if (kRefill) load_group(b + 1, k);
            }
        }
    };
    if (nbat > 0) {                                                  // uniform per wave; no barrier inside
#pragma unroll
        for (int k = 0; k < GB; ++k) load_group(0, k);
        load_act(0);
        store_act();
        for (int b = 0; b + 1 < nbat; ++b) {
            load_act(b + 1);
            multiply(std::true_type{}, b, GB);
            store_act();
        }
        multiply(std::false_type{}, nbat - 1, u1 - u0 - (nbat - 1) * GB);
    }
    // a wave's partial sums go where its activations were (its own region, it is done with them)
    auto red = [&](int w) { return reinterpret_cast<float *>(lds + kQDownFixed + (size_t)w * region) + lane * 4 * TILES; };
#pragma unroll
    for (int tl = 0; tl < TILES; ++tl)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) red(wave)[4 * tl + rr] = c[tl][rr];
    __syncthreads();
    if (wave < TILES && i < T) {                                     // wave tl finishes tile tl
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            float v = red(0)[4 * wave + rr];
#pragma unroll
            for (int w = 1; w < WAVES; ++w) v += red(w)[4 * wave + rr];
            y[(size_t)i * d + j0 + 16 * wave + 4 * q + rr] = f32_to_bf16(v);
        }
    }
}

bool q4_mfma_path_supported(int T, int d, int G, int gs)
{
    return T >= 2 && T <= 16 && gs == kQ4Block && d % (kQBatch * kQ4Block) == 0 && d <= 8192 && G <= 256;
}

hipError_t launch_ffn_q4_mfma(const bf16_t *x, int T, int d, int G, const Q4Weights &w, const uint8_t *mask,
                              bf16_t *y, const DecodeScratch &ws, hipStream_t s, int rank, const AheadArgs *ahead,
                              bool *ahead_fused)
{
    const int ffn = G * kQ4Block;
    bf16_t *act = reinterpret_cast<bf16_t *>(ws.act);
    const AheadArgs *ah = (ahead && ahead_fused) ? ahead : nullptr;
    if (ahead_fused) *ahead_fused = ah != nullptr;
    AheadPredDev ap = ahead_pred_dev(ah);
    ap.r = rank;                                            // the work is shaped by it whether or not the rows ride along
    const int n_mask = ah ? T : 0;
    const AheadDev nx = ah ? ahead_dev(*ah) : AheadDev{};
    // the predictor rows ride inside the same workgroups: ap.n_pred only says whether there are any
    if ((size_t)T * d * sizeof(bf16_t) <= (size_t)q_x_bytes(4))
        launch_timed("gate_up_q4_mt", gate_up_q4_mt<4>, dim3(q_gate_up_blocks(4)), dim3(256), s, x, T, d, G, w.gate_codes,
                     w.gate_scales, w.up_codes, w.up_scales, mask, act, ffn, ap);
    else
        launch_timed("gate_up_q4_mt", gate_up_q4_mt<8>, dim3(q_gate_up_blocks(8)), dim3(512), s, x, T, d, G, w.gate_codes,
                     w.gate_scales, w.up_codes, w.up_scales, mask, act, ffn, ap);
    // long rows: 32 rows to a workgroup of eight waves, so that the activations are read half as often
    const bool wide = d >= 8192 && d % 32 == 0;
#define HALO_DOWN_Q4(TM, TILES, WAVES, GB)                                                                       \
    do {                                                                                                         \
        static const hipError_t lds_ok = hipFuncSetAttribute(                                                    \
            reinterpret_cast<const void *>(down_q4_mt<TM, TILES, WAVES, GB>), hipFuncAttributeMaxDynamicSharedMemorySize, \
            (int)q_down_lds_bytes(16, WAVES, GB, TILES));                                                               \
        if (lds_ok != hipSuccess) return lds_ok;                                                                 \
        down_q4_mt<TM, TILES, WAVES, GB><<<dim3(d / (16 * TILES) + n_mask), dim3(WAVES * 64), q_down_lds_bytes(T, WAVES, GB, TILES), s>>>( \
            T, d, G, w.down_codes, w.down_scales, mask, act, ffn, y, n_mask, nx);                                \
    } while (0)
    if (wide) {
        if (T <= 4)
            HALO_DOWN_Q4(4, 2, 8, 2);
        else if (T <= 8)
            HALO_DOWN_Q4(8, 2, 8, 2);
        else
            HALO_DOWN_Q4(16, 2, 8, 2);
    } else {
        if (T <= 4)
            HALO_DOWN_Q4(4, 1, 4, 4);
        else if (T <= 8)
            HALO_DOWN_Q4(8, 1, 4, 4);
        else
            HALO_DOWN_Q4(16, 1, 4, 4);
    }
#undef HALO_DOWN_Q4
    return hipGetLastError();
}

}  // namespace halo
