// Group-sparse SwiGLU FFN for a few tokens (2 <= T <= 16) on the matrix cores, bf16.
//
// The block is still bound by streaming the surviving groups' weights from HBM (every
// weight byte is used T times), so the layout of the work follows the memory stream and
// the matrix instruction is only a cheap way to apply one 16-byte weight piece to all
// tokens at once (v_mfma_f32_16x16x32_bf16: 16 weight rows x 16 tokens x 32 elements).
//
//   gate/up : each wave owns a contiguous run of the union's neurons (runs differ by at
//             most one), cut into tiles of <= 16 rows, and sweeps the rows in 512-element
//             chunks; the token fragments are read from x directly (it is small and stays
//             in cache).  act[t][n] = mask ? SiLU(gate)*up : 0 is stored in bf16.
//   down    : Wd is group-blocked, Wd[g][j][m]; a workgroup owns a run of consecutive output
//             rows j (one workgroup per compute unit where the row count allows), its four
//             waves split the union's groups, partial tiles are added through LDS and y is
//             written directly.
// Operand layout of the instruction (wave64): A lane l holds row l%16, elements
// 8*(l/16)..+7 of the 32; B lane l holds column l%16, same elements; D lane l holds
// column l%16, rows 4*(l/16)..+3.  Rows are neurons (or outputs j), columns are tokens.
#include "kernels.hpp"
#include "mask_device.hpp"
#include "mask_words.hpp"

namespace halo {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4_t mfma16(const u32x4 &a, const u32x4 &b, const f32x4_t &c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// Both kernels fetch weights the way the one-token path does -- a wave reads 1 KiB of
// consecutive bytes per instruction, non-temporal -- and re-shape them into the matrix
// instruction's operand layout through a private LDS region of the wave (16-byte writes in
// row order, 16-byte reads in operand order; rows are padded by 16 bytes so that the reads
// of a 16-lane group hit distinct banks).  Letting each lane fetch its own operand piece
// instead touches 4x more cache lines per instruction and ran at 40 % of this.
constexpr int kChunk = 512;                 // row elements per fetch instruction (64 lanes x 8)
constexpr int kChunkRow = kChunk + 8;       // padded LDS row, elements

// grid: any number of 256-thread workgroups; LDS = 4 waves x 16 rows x 1040 B.
// Waves take contiguous runs of about 12 neurons (fewer waves work when the union is small, so
// that a tile is not mostly padding); the gate rows of a chunk are multiplied while the up
// rows of the same chunk are in flight, and the up rows while the next chunk's gate rows are.
struct RowRegs {
    u32x4 v[16];
};

// UNION_IN_KERNEL (T <= 16, G <= 256): the union list is built here from the tokens' masks instead of
// being read from memory (ulist / meta written by an earlier launch).
template <bool UNION_IN_KERNEL>
__global__ __launch_bounds__(256) void gate_up_mt(
    const bf16_t *__restrict__ x, int T, int d, int G, int gs, const bf16_t *__restrict__ Wg,
    const bf16_t *__restrict__ Wu, const uint8_t *__restrict__ mask, const int32_t *__restrict__ ulist_mem,
    const int32_t *__restrict__ meta, bf16_t *__restrict__ act, int act_stride, AheadPredDev ap)
{
    __shared__ __attribute__((aligned(16))) bf16_t sW[4][16 * kChunkRow];
    __shared__ int s_list[256];
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
    bf16_t *my = sW[wave];
    const int32_t *ulist = ulist_mem;
    long long total;
    if (UNION_IN_KERNEL) {
        const MaskWords uw = load_union_words<16>(mask, T, G, lane);
        if (wave == 0) write_group_list(uw, lane, s_list);
        __syncthreads();
        total = (long long)uw.count * gs;
        ulist = s_list;
    } else {
        total = (long long)meta[0] * gs;
    }
    int nw = (gridDim.x - ap.n_pred) * 4;
    const long long want = (total + 11) / 12;
    if (want < nw) nw = want < 1 ? 1 : (int)want;
    const int w = (blockIdx.x - ap.n_pred) * 4 + wave;
    if (w >= nw) return;
    const int n0 = (int)(total * w / nw), n1 = (int)(total * (w + 1) / nw);
    const int L = n1 - n0;
    if (L <= 0) return;
    const int ntile = (L + 15) / 16;
    const int i = lane & 15, q = lane >> 4;
    const int tok = i < T ? i : T - 1;                      // columns >= T repeat the last token, unused
    const bf16_t *xrow = x + (size_t)tok * d + q * 8;
    const int nck = (d + kChunk - 1) / kChunk;              // the last chunk may be 128, 256 or 384 wide
    for (int tile = 0; tile < ntile; ++tile) {
        const int r0 = n0 + (int)((long long)L * tile / ntile);
        const int r1 = n0 + (int)((long long)L * (tile + 1) / ntile);     // r1 - r0 <= 16
        const int cnt = r1 - r0;
        size_t wrow[16];                                    // wave-uniform
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const int n = k < cnt ? r0 + k : r1 - 1;
            const int u = n / gs;
            wrow[k] = ((size_t)ulist[u] * gs + (n - u * gs)) * d;
        }
        auto width_of = [&](int c) { return min(kChunk, d - c * kChunk); };
        auto fetch = [&](RowRegs &r, const bf16_t *W, int c) {
            const bool on = lane * 8 < width_of(c);
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                r.v[k] = u32x4{0u, 0u, 0u, 0u};
                if (k < cnt && on)
                    r.v[k] = __builtin_nontemporal_load(
                        reinterpret_cast<const u32x4 *>(W + wrow[k] + c * kChunk + lane * 8));
            }
        };
        auto fetch_x = [&](u32x4 (&b)[16], int c) {
            const int steps = width_of(c) / 32;
#pragma unroll
            for (int s = 0; s < 16; ++s)
                b[s] = s < steps ? *reinterpret_cast<const u32x4 *>(xrow + c * kChunk + s * 32)
                                 : u32x4{0u, 0u, 0u, 0u};
        };
        auto multiply = [&](const RowRegs &r, const u32x4 (&b)[16], int c, f32x4_t &acc) {
            const int steps = width_of(c) / 32;
#pragma unroll
            for (int k = 0; k < 16; ++k)
                *reinterpret_cast<u32x4 *>(my + k * kChunkRow + lane * 8) = r.v[k];
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                if (s < steps) {
                    const u32x4 a = *reinterpret_cast<const u32x4 *>(my + i * kChunkRow + s * 32 + q * 8);
                    acc = mfma16(a, b[s], acc);
                }
            }
        };
        f32x4_t cg = {0.f, 0.f, 0.f, 0.f}, cu = {0.f, 0.f, 0.f, 0.f};
        RowRegs R0, R1;
        u32x4 b[16];
        fetch_x(b, 0);
        fetch(R0, Wg, 0);
        for (int c = 0; c + 1 < nck; ++c) {
            fetch(R1, Wu, c);
            multiply(R0, b, c, cg);
            fetch(R0, Wg, c + 1);
            multiply(R1, b, c, cu);
            fetch_x(b, c + 1);
        }
        fetch(R1, Wu, nck - 1);
        multiply(R0, b, nck - 1, cg);
        multiply(R1, b, nck - 1, cu);
        // D: column = token i, rows 4q..4q+3 of the tile
        if (i < T) {
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int nn = r0 + 4 * q + rr;
                if (nn < r1) {
                    const int g = ulist[nn / gs];
                    const float v = mask[(size_t)i * G + g] ? silu_mul(cg[rr], cu[rr]) : 0.0f;
                    act[(size_t)i * act_stride + nn] = f32_to_bf16(v);
                }
            }
        }
    }
}

// grid: d / (4 LD) workgroups of 256 threads; group size 128.  A workgroup owns 4 LD consecutive output
// rows; a group's tile of Wd for them is LD KiB of consecutive bytes, fetched by LD instructions.
// LD is chosen by the host so that the grid is one workgroup per compute unit where the row count
// allows it (d a multiple of 1024: LD = d / 1024, 256 workgroups).  A compute unit draws from memory at
// a bounded rate whatever the number of workgroups on it, so a grid of 320 workgroups (d = 5120 in
// 16-row tiles) runs as long as the compute units that hold two of them: 19 us against 12.
constexpr int kTileRow = 128 + 8;           // padded LDS row, elements

template <int LD>
struct DownMtShared {
    static constexpr int kTiles = (LD + 3) / 4;             // 16-row tiles of the matrix instruction
    static constexpr int kGroups = LD <= 4 ? 3 : 2;         // groups per batch of registers
    __attribute__((aligned(16))) bf16_t sT[4][kGroups][16 * kTiles * kTileRow];
    int s_list[256];
};

// UNION_IN_KERNEL: as in gate_up_mt.  The first n_mask workgroups do not project: each computes the
// next block's scores, ranking and mask for one token (n_mask = 0: nobody does).
template <bool UNION_IN_KERNEL, int LD>
__global__ __launch_bounds__(256) void down_mt(
    int T, int d, int G, const bf16_t *__restrict__ Wd, const uint8_t *__restrict__ mask,
    const int32_t *__restrict__ ulist_mem, const int32_t *__restrict__ meta,
    const bf16_t *__restrict__ act, int act_stride, bf16_t *__restrict__ y, int n_mask, AheadDev nx)
{
    constexpr int gs = 128;
    using Shared = DownMtShared<LD>;
    constexpr int kTiles = Shared::kTiles, kGroups = Shared::kGroups;
    constexpr size_t kLds = sizeof(Shared) > sizeof(MaskShared) ? sizeof(Shared) : sizeof(MaskShared);
    __shared__ __attribute__((aligned(16))) unsigned char lds[kLds];
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
    Shared &sh = *reinterpret_cast<Shared *>(lds);
    auto &sT = sh.sT;
    auto &s_list = sh.s_list;
    // the waves' partial sums meet in LDS at the end; each wave parks its own at the start of its own
    // tile region, which it has finished reading by then
    auto red = [&](int w) { return reinterpret_cast<float(*)[64][4]>(&sT[w][0][0]); };
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int i = lane & 15, q = lane >> 4;
    const int j0 = (blockIdx.x - n_mask) * (4 * LD);
    int n_u;
    const int32_t *ulist = ulist_mem;
    if (UNION_IN_KERNEL) {
        const MaskWords uw = load_union_words<16>(mask, T, G, lane);
        if (wave == 0) write_group_list(uw, lane, s_list);
        __syncthreads();
        n_u = uw.count;
        ulist = s_list;
    } else {
        n_u = meta[0];
    }
    const int u0 = n_u * wave / 4, u1 = n_u * (wave + 1) / 4;
    const int tok = i < T ? i : T - 1;
    const bf16_t *arow = act + (size_t)tok * act_stride + q * 8;
    const size_t gstride = (size_t)d * gs;
    const bf16_t *wtile = Wd + (size_t)j0 * gs + lane * 8;          // + n*512 elements for instruction n
    f32x4_t c[kTiles];
#pragma unroll
    for (int tt = 0; tt < kTiles; ++tt) c[tt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    // Two batches of registers: the next batch of groups is requested before the current one is
    // re-shaped and multiplied, so the wave always has loads outstanding (with one batch, every
    // batch was a memory round trip of its own).
    struct Batch {
        u32x4 r[kGroups][LD], b[kGroups][4];
    };
    auto request = [&](Batch &t, int ub) {
#pragma unroll
        for (int k = 0; k < kGroups; ++k) {
            const int u = ub + k < u1 ? ub + k : u1 - 1;             // past the end: in-range duplicate
            const bf16_t *pw = wtile + ulist[u] * gstride;
            const bf16_t *pa = arow + (size_t)u * gs;
#pragma unroll
            for (int n = 0; n < LD; ++n)
                t.r[k][n] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(pw + n * 512));
#pragma unroll
            for (int s = 0; s < 4; ++s) t.b[k][s] = *reinterpret_cast<const u32x4 *>(pa + s * 32);
        }
    };
    auto consume = [&](const Batch &t, int ub) {
        // instruction n, lane l holds row 4n + l/16, elements (l%16)*8..+7
#pragma unroll
        for (int k = 0; k < kGroups; ++k)
#pragma unroll
            for (int n = 0; n < LD; ++n)
                *reinterpret_cast<u32x4 *>(&sT[wave][k][(4 * n + q) * kTileRow + i * 8]) = t.r[k][n];
        // rows of the last tile past 4 LD hold whatever LDS held: a row of the product depends on its
        // own row of the operand only, and those rows are never stored
#pragma unroll
        for (int k = 0; k < kGroups; ++k) {
            if (ub + k < u1) {
#pragma unroll
                for (int tt = 0; tt < kTiles; ++tt)
#pragma unroll
                    for (int s = 0; s < 4; ++s) {
                        const u32x4 a = *reinterpret_cast<const u32x4 *>(
                            &sT[wave][k][(16 * tt + i) * kTileRow + s * 32 + q * 8]);
                        c[tt] = mfma16(a, t.b[k][s], c[tt]);
                    }
            }
        }
    };
    if (u0 < u1) {
        Batch P, Q;
        request(P, u0);
        int ub = u0;
        while (ub + 2 * kGroups < u1) {
            request(Q, ub + kGroups);
            consume(P, ub);
            request(P, ub + 2 * kGroups);
            consume(Q, ub + kGroups);
            ub += 2 * kGroups;
        }
        if (ub + kGroups < u1) {
            request(Q, ub + kGroups);
            consume(P, ub);
            consume(Q, ub + kGroups);
        } else {
            consume(P, ub);
        }
    }
#pragma unroll
    for (int tt = 0; tt < kTiles; ++tt)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) red(wave)[tt][lane][rr] = c[tt][rr];
    __syncthreads();
    if (wave == 0 && i < T) {
#pragma unroll
        for (int tt = 0; tt < kTiles; ++tt)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int row = 16 * tt + 4 * q + rr;
                if (row < 4 * LD) {
                    const float v = ((red(0)[tt][lane][rr] + red(1)[tt][lane][rr]) + red(2)[tt][lane][rr]) +
                                    red(3)[tt][lane][rr];
                    y[(size_t)i * d + j0 + row] = f32_to_bf16(v);
                }
            }
    }
}

// LD = d / 1024 where d is a multiple of 1024 up to 8192 (one workgroup per compute unit), else 16-row
// workgroups
template <bool UNION_IN_KERNEL>
static void launch_down_mt(int T, int d, int G, const bf16_t *Wd, const uint8_t *mask, const int32_t *ulist,
                           const int32_t *meta, const bf16_t *act, int act_stride, bf16_t *y, int n_mask,
                           const AheadDev &nx, hipStream_t s)
{
#define HALO_DOWN_MT_CASE(LD_)                                                                                    \
    case LD_:                                                                                                     \
        down_mt<UNION_IN_KERNEL, LD_><<<dim3(d / (4 * LD_) + n_mask), dim3(256), 0, s>>>(T, d, G, Wd, mask, ulist, \
                                                                                         meta, act, act_stride, y, \
                                                                                         n_mask, nx);              \
        break;
    switch ((d % 1024 == 0 && d >= 2048 && d <= 8192) ? d / 1024 : 4) {
        HALO_DOWN_MT_CASE(2)
        HALO_DOWN_MT_CASE(3)
        HALO_DOWN_MT_CASE(4)
        HALO_DOWN_MT_CASE(5)
        HALO_DOWN_MT_CASE(6)
        HALO_DOWN_MT_CASE(7)
        HALO_DOWN_MT_CASE(8)
    }
#undef HALO_DOWN_MT_CASE
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
bool mfma_path_supported(int T, int d, int gs)
{
    return T >= 2 && T <= 16 && d % 128 == 0 && gs == 128;
}

hipError_t launch_ffn_mfma(const bf16_t *x, int T, int d, int G, int gs, const bf16_t *Wg,
                           const bf16_t *Wu, const bf16_t *Wd, const uint8_t *mask, bf16_t *y,
                           const DecodeScratch &ws, hipStream_t s, const AheadArgs *ahead, bool *ahead_fused)
{
    const int ffn = G * gs;
    bf16_t *act = reinterpret_cast<bf16_t *>(ws.act);
    if (ahead_fused) *ahead_fused = false;
    if (G <= 256) {
        // The union of the tokens' groups is built inside the kernels: no union launch, no list in
        // memory.  The next block's prediction can ride along: its first layer in spare workgroups
        // of the gate/up launch, its second layer + ranking + mask (a workgroup per token) in the
        // down-projection launch.
        const AheadArgs *ah = (ahead && ahead_fused) ? ahead : nullptr;
        if (ah) *ahead_fused = true;
        const AheadPredDev ap = ahead_pred_dev(ah);
        const int n_mask = ah ? T : 0;
        const AheadDev nx = ah ? ahead_dev(*ah) : AheadDev{};
        if (few_path_supported(T, d, G, gs)) {
            // up to four tokens: rows streamed as in the one-token path
            hipError_t e = launch_gate_up_few(x, T, d, G, gs, Wg, Wu, mask, act, ffn, s, ap);
            if (e != hipSuccess) return e;
        } else {
            launch_timed("gate_up_mt", gate_up_mt<true>, dim3(256 + ap.n_pred), dim3(256), s, x, T, d, G, gs, Wg, Wu,
                         mask, (const int32_t *)nullptr, (const int32_t *)nullptr, act, ffn, ap);
        }
        launch_down_mt<true>(T, d, G, Wd, mask, nullptr, nullptr, act, ffn, y, n_mask, nx, s);
        return hipGetLastError();
    }
    hipError_t e = launch_union(mask, T, G, ws.ulist, ws.meta, s);
    if (e != hipSuccess) return e;
    // one workgroup per compute unit (the kernel holds two row batches in registers, one wave per SIMD)
    launch_timed("gate_up_mt", gate_up_mt<false>, dim3(256), dim3(256), s, x, T, d, G, gs, Wg, Wu, mask,
                 (const int32_t *)ws.ulist, (const int32_t *)ws.meta, act, ffn, AheadPredDev{nullptr, nullptr, nullptr, 0, 0});
    launch_down_mt<false>(T, d, G, Wd, mask, ws.ulist, ws.meta, act, ffn, y, 0, AheadDev{}, s);
    return hipGetLastError();
}

}  // namespace halo
