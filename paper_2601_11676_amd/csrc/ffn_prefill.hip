// Group-sparse SwiGLU FFN for many tokens (prefill) on the matrix cores, bf16.
//
// With hundreds of tokens the block is a dense contraction per neuron group, but only over
// the tokens that keep the group (paper Sec. II-A: groups are independent until the merge;
// Sec. III-B.3: each token has its own surviving set).  Three kernels:
//
//   group_tokens : for every group, the ascending list of tokens that keep it, and for
//                  every (token, group) the token's slot in that list (-1 = not kept).
//   gate_up_pf   : one workgroup = 64 neurons of one group x up to 128 of the group's
//                  tokens.  The 128 weight rows (64 gate + 64 up) are staged through LDS once
//                  per 64-element K step and shared by the four waves; each wave owns 32
//                  tokens and loads their x rows (gathered by the token list) straight into
//                  registers as the B operand.  A group's weights are read once from HBM and
//                  once more from cache per further 128 tokens.
//                  act[g][slot][m] = SiLU(gate) * up in bf16.
//   down_pf      : output-stationary: one workgroup = 128 tokens x 64 outputs, walking all
//                  groups (Wd tiles through LDS, activation rows gathered into registers); a
//                  token that does not keep a group feeds zeros, so it contributes exactly
//                  nothing, and every y element has exactly one writer (no atomics).
//
// v_mfma_f32_16x16x32_bf16 operand layout as in ffn_mfma.hip: A lane l = row l%16, elements
// 8*(l/16)..+7; B lane l = column l%16, same elements; D lane l = column l%16, rows 4*(l/16)..+3.
#include "kernels.hpp"

namespace halo {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4_t mfma16p(const u32x4 &a, const u32x4 &b, const f32x4_t &c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// ---------------------------------------------------------------------------
// token lists: grid = G workgroups of 256 threads
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void group_tokens_kernel(const uint8_t *__restrict__ mask, int T, int G,
                                                           int32_t *__restrict__ tok_list,
                                                           int32_t *__restrict__ tok_cnt,
                                                           int32_t *__restrict__ slot)
{
    __shared__ int s_wave[4];
    __shared__ int s_base;
    const int g = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if (tid == 0) s_base = 0;
    __syncthreads();
    for (int t0 = 0; t0 < T; t0 += 256) {
        const int t = t0 + tid;
        const bool keep = t < T && mask[(size_t)t * G + g] != 0;
        const unsigned long long b = __ballot(keep);
        if (lane == 0) s_wave[wave] = __popcll(b);
        __syncthreads();
        int before = s_base;
        for (int k = 0; k < wave; ++k) before += s_wave[k];
        const int pos = before + __popcll(b & ((1ull << lane) - 1ull));
        if (keep) tok_list[(size_t)g * T + pos] = t;
        if (t < T) slot[(size_t)t * G + g] = keep ? pos : -1;
        __syncthreads();
        if (tid == 0) s_base += s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
        __syncthreads();
    }
    if (tid == 0) tok_cnt[g] = s_base;
}

// ---------------------------------------------------------------------------
// gate/up: grid (G * gs/NB, ceil(T/128)), 256 threads
// ---------------------------------------------------------------------------
constexpr int kKS = 64;             // K elements per LDS stage (32 and 128 measured slower)
constexpr int kARow = kKS + 8;      // padded LDS row (elements): rows start 16 bytes apart in bank space
constexpr int kKH = kKS / 32;       // matrix-instruction K steps per stage

// TT = 16-token tiles per wave (a workgroup covers 4 * TT * 16 tokens of the group's list);
// NB = neurons per workgroup (32 or 64).  Both operands go through LDS: the 2*NB weight rows and
// the workgroup's gathered x rows are fetched with coalesced 128-byte row segments (eight lanes
// per row), parked in registers for a stage and written to the other LDS buffer, so both are
// requested two stages before the matrix instructions read them.  (Letting each lane fetch
// its own x operand piece straight from memory touched 16 rows per instruction and could only
// be requested one stage ahead; waves spent more than half their time waiting.)
template <int TT, int NB>
__global__ __launch_bounds__(256) void gate_up_pf(
    const bf16_t *__restrict__ x, int T, int d, int gs, const bf16_t *__restrict__ Wg,
    const bf16_t *__restrict__ Wu, const int32_t *__restrict__ tok_list,
    const int32_t *__restrict__ tok_cnt, bf16_t *__restrict__ act)
{
    constexpr int HT = NB / 16;                              // 16-row tiles per matrix
    constexpr int RPP = 256 / (kKS / 8);                     // rows staged per pass (kKS/8 threads per row)
    constexpr int NP = NB / RPP;                             // staging passes per weight matrix
    constexpr int kTok = 4 * TT * 16;                        // tokens per workgroup
    constexpr int NPX = kTok / RPP;                          // staging passes for the x tile
    __shared__ __attribute__((aligned(16))) bf16_t sA[2][2 * NB * kARow];
    __shared__ __attribute__((aligned(16))) bf16_t sX[2][kTok * kARow];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int i16 = lane & 15, q = lane >> 4;
    const int per_group = gs / NB;
    const int g = blockIdx.x / per_group, nt = blockIdx.x - g * per_group;
    const int cnt = tok_cnt[g];
    const int c0 = blockIdx.y * kTok;
    if (c0 >= cnt) return;                                   // uniform for the workgroup
    const int32_t *list = tok_list + (size_t)g * T;
    // staging role of this thread: kKS/8 threads share a row's segment of a stage; per pass the
    // thread takes gate row sr + RPP*p and up row sr + RPP*p (LDS rows r and NB + r), piece sp,
    // and x row (= token slot) sr + RPP*p of the workgroup's tile
    const int sr = tid / (kKS / 8), sp = tid % (kKS / 8);
    const size_t neuron0 = (size_t)g * gs + nt * NB;
    const bf16_t *wsrc_g = Wg + (neuron0 + sr) * d + sp * 8;
    const bf16_t *wsrc_u = Wu + (neuron0 + sr) * d + sp * 8;
    const int dst_off = sr * kARow + sp * 8;
    const bf16_t *xsrc[NPX];
#pragma unroll
    for (int p = 0; p < NPX; ++p) {
        int sl = c0 + sr + RPP * p;
        sl = sl < cnt ? sl : cnt - 1;                        // past the end: a valid duplicate, never stored
        xsrc[p] = x + (size_t)list[sl] * d + sp * 8;
    }

    f32x4_t acc[2 * HT][TT];
#pragma unroll
    for (int mt = 0; mt < 2 * HT; ++mt)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) acc[mt][tt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    struct Stage {
        u32x4 g[NP], u[NP], x[NPX];
    };
    auto load_stage = [&](int k0, Stage &r) {
#pragma unroll
        for (int p = 0; p < NPX; ++p) r.x[p] = *reinterpret_cast<const u32x4 *>(xsrc[p] + k0);
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            r.g[p] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wsrc_g + (size_t)p * RPP * d + k0));
            r.u[p] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wsrc_u + (size_t)p * RPP * d + k0));
        }
    };
    auto store_stage = [&](int buf, const Stage &r) {
#pragma unroll
        for (int p = 0; p < NPX; ++p) *reinterpret_cast<u32x4 *>(sX[buf] + dst_off + p * RPP * kARow) = r.x[p];
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            *reinterpret_cast<u32x4 *>(sA[buf] + dst_off + p * RPP * kARow) = r.g[p];
            *reinterpret_cast<u32x4 *>(sA[buf] + dst_off + (NB + p * RPP) * kARow) = r.u[p];
        }
    };
    auto compute = [&](int buf) {
        const bf16_t *a_lds = sA[buf], *x_lds = sX[buf];
#pragma unroll
        for (int kh = 0; kh < kKH; ++kh) {
            u32x4 a[2 * HT], b[TT];
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
                b[tt] = *reinterpret_cast<const u32x4 *>(x_lds + ((wave * TT + tt) * 16 + i16) * kARow + kh * 32 + q * 8);
#pragma unroll
            for (int mt = 0; mt < 2 * HT; ++mt)
                a[mt] = *reinterpret_cast<const u32x4 *>(a_lds + (mt * 16 + i16) * kARow + kh * 32 + q * 8);
#pragma unroll
            for (int mt = 0; mt < 2 * HT; ++mt)
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) acc[mt][tt] = mfma16p(a[mt], b[tt], acc[mt][tt]);
        }
    };

    // software pipeline over K (an even number of stages, d % 128 == 0).  Top of an even stage s:
    // LDS buffer 0 holds stage s; r1 = stage s+1 is in flight.
    const int nstage = d / kKS;
    Stage r0, r1;
    load_stage(0, r0);
    load_stage(kKS, r1);
    store_stage(0, r0);
    __syncthreads();
    int s = 0;
    for (; s + 2 < nstage; s += 2) {
        load_stage((s + 2) * kKS, r0);
        compute(0);
        store_stage(1, r1);
        __syncthreads();
        load_stage((s + 3) * kKS, r1);
        compute(1);
        store_stage(0, r0);
        __syncthreads();
    }
    compute(0);
    store_stage(1, r1);
    __syncthreads();
    compute(1);

    // D: column = token i16 of tile tt, rows 4q..4q+3 of a neuron tile (tiles 0..HT-1 gate, HT.. up)
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        const int sl = c0 + (wave * TT + tt) * 16 + i16;
        if (sl < cnt) {
#pragma unroll
            for (int mt = 0; mt < HT; ++mt) {
                uint32_t lo = (uint32_t)f32_to_bf16(silu_mul(acc[mt][tt][0], acc[mt + HT][tt][0])) |
                              ((uint32_t)f32_to_bf16(silu_mul(acc[mt][tt][1], acc[mt + HT][tt][1])) << 16);
                uint32_t hi = (uint32_t)f32_to_bf16(silu_mul(acc[mt][tt][2], acc[mt + HT][tt][2])) |
                              ((uint32_t)f32_to_bf16(silu_mul(acc[mt][tt][3], acc[mt + HT][tt][3])) << 16);
                bf16_t *dst = act + ((size_t)g * T + sl) * gs + nt * NB + mt * 16 + 4 * q;
                *reinterpret_cast<uint2 *>(dst) = make_uint2(lo, hi);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// down: grid (d/64, ceil(T/128)), 256 threads; group size 128
// ---------------------------------------------------------------------------
// A workgroup owns 128 tokens x 64 outputs and walks the groups.  The group's 64 x 128 tile of
// Wd is 16 KiB of consecutive bytes: it is fetched once per workgroup with coalesced loads,
// staged through LDS and shared by the four waves (each wave loading its own operand pieces
// cost four times the L1 traffic and ran at 8 % of the matrix peak).  The activation rows are
// private to a wave (its 32 tokens), gathered by slot straight into registers; a token that
// does not keep the group gets a zero fragment and so contributes exactly nothing.
constexpr int kWdRow = 128 + 8;     // padded LDS row of the Wd tile, elements

struct ActFrags {
    u32x4 b[4][2];                  // [k step][token tile]
};

__global__ __launch_bounds__(256) void down_pf(
    int T, int d, int G, const bf16_t *__restrict__ Wd, const int32_t *__restrict__ slot,
    const bf16_t *__restrict__ act, bf16_t *__restrict__ y)
{
    constexpr int gs = 128;
    __shared__ __attribute__((aligned(16))) bf16_t sWd[2][64 * kWdRow];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int i16 = lane & 15, q = lane >> 4;
    const int j0 = blockIdx.x * 64;
    const int t0 = blockIdx.y * 128 + wave * 32;       // may be >= T for the last workgroup's upper waves:
                                                        // those waves still stage Wd and meet the barriers
    const int32_t *sl0, *sl1;
    {
        const int ta = t0 + i16, tb = t0 + 16 + i16;
        sl0 = slot + (size_t)(ta < T ? ta : T - 1) * G;          // duplicates of a valid token, never stored
        sl1 = slot + (size_t)(tb < T ? tb : T - 1) * G;
    }
    f32x4_t acc[4][2];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) acc[mt][tt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const size_t gstride = (size_t)d * gs;
    // staging role: the tile is 1024 pieces of 16 bytes; this thread moves pieces tid + 256 n
    const bf16_t *wsrc = Wd + (size_t)j0 * gs + tid * 8;
    int wdst[4];
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        const int p = tid + 256 * n;
        wdst[n] = (p >> 4) * kWdRow + (p & 15) * 8;
    }
    auto load_w = [&](u32x4 (&r)[4], int g) {
#pragma unroll
        for (int n = 0; n < 4; ++n)
            r[n] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wsrc + g * gstride + n * 2048));
    };
    auto store_w = [&](bf16_t *buf, const u32x4 (&r)[4]) {
#pragma unroll
        for (int n = 0; n < 4; ++n) *reinterpret_cast<u32x4 *>(buf + wdst[n]) = r[n];
    };
    auto load_act = [&](ActFrags &f, int g, int s0, int s1) {
        const bf16_t *pb0 = act + ((size_t)g * T + (s0 < 0 ? 0 : s0)) * gs + q * 8;
        const bf16_t *pb1 = act + ((size_t)g * T + (s1 < 0 ? 0 : s1)) * gs + q * 8;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const u32x4 v0 = *reinterpret_cast<const u32x4 *>(pb0 + ks * 32);
            const u32x4 v1 = *reinterpret_cast<const u32x4 *>(pb1 + ks * 32);
            f.b[ks][0] = s0 < 0 ? u32x4{0u, 0u, 0u, 0u} : v0;
            f.b[ks][1] = s1 < 0 ? u32x4{0u, 0u, 0u, 0u} : v1;
        }
    };
    auto multiply = [&](const bf16_t *buf, const ActFrags &f) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            u32x4 a[4];
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
                a[mt] = *reinterpret_cast<const u32x4 *>(buf + (mt * 16 + i16) * kWdRow + ks * 32 + q * 8);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
                acc[mt][0] = mfma16p(a[mt], f.b[ks][0], acc[mt][0]);
                acc[mt][1] = mfma16p(a[mt], f.b[ks][1], acc[mt][1]);
            }
        }
    };
    // groups in pairs.  A group's Wd tile travels global -> registers -> LDS two groups ahead of its
    // use, its activation fragments one group ahead, the slots (which the fragment addresses depend
    // on) one group further.  Loads past the last group repeat the last group (harmless).
    // Top of an even step g: sWd[0] holds W(g); rw1 = W(g+1) and F0 = act(g) are in flight;
    // (s0, s1) are the slots of group g+1.
    auto cl = [&](int g) { return g < G ? g : G - 1; };
    u32x4 rw0[4], rw1[4];
    ActFrags F0, F1;
    int s0 = sl0[0], s1 = sl1[0];
    load_w(rw0, 0);
    load_act(F0, 0, s0, s1);
    load_w(rw1, cl(1));
    s0 = sl0[cl(1)]; s1 = sl1[cl(1)];
    int n0 = sl0[cl(2)], n1 = sl1[cl(2)];       // slots of group g+2
    store_w(sWd[0], rw0);
    __syncthreads();
    int g = 0;
    for (; g + 1 < G; g += 2) {
        load_act(F1, cl(g + 1), s0, s1);
        load_w(rw0, cl(g + 2));
        s0 = n0; s1 = n1;                       // slots of group g+2
        n0 = sl0[cl(g + 3)]; n1 = sl1[cl(g + 3)];
        multiply(sWd[0], F0);
        store_w(sWd[1], rw1);
        __syncthreads();
        load_act(F0, cl(g + 2), s0, s1);
        load_w(rw1, cl(g + 3));
        s0 = n0; s1 = n1;                       // slots of group g+3
        n0 = sl0[cl(g + 4)]; n1 = sl1[cl(g + 4)];
        multiply(sWd[1], F1);
        store_w(sWd[0], rw0);
        __syncthreads();
    }
    if (g < G) multiply(sWd[0], F0);            // an odd number of groups: the last one
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
        const int t = t0 + tt * 16 + i16;
        if (t < T) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
                uint32_t lo = (uint32_t)f32_to_bf16(acc[mt][tt][0]) | ((uint32_t)f32_to_bf16(acc[mt][tt][1]) << 16);
                uint32_t hi = (uint32_t)f32_to_bf16(acc[mt][tt][2]) | ((uint32_t)f32_to_bf16(acc[mt][tt][3]) << 16);
                *reinterpret_cast<uint2 *>(y + (size_t)t * d + j0 + mt * 16 + 4 * q) = make_uint2(lo, hi);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
bool prefill_path_supported(int T, int d, int gs)
{
    return T > 1 && d % 128 == 0 && gs == 128;
}

hipError_t launch_ffn_prefill(const bf16_t *x, int T, int d, int G, int gs, const bf16_t *Wg,
                              const bf16_t *Wu, const bf16_t *Wd, const uint8_t *mask, bf16_t *y,
                              const DecodeScratch &ws, hipStream_t s)
{
    bf16_t *act = reinterpret_cast<bf16_t *>(ws.act);
    group_tokens_kernel<<<dim3(G), dim3(256), 0, s>>>(mask, T, G, ws.tok_list, ws.tok_cnt, ws.slot);
    // 128 tokens x 64 neurons per workgroup.  Measured on the 512-token LLaMA-7B shape: 32 neurons
    // 169 us, 64 neurons 120 us, the whole group with 64 tokens 151 us.
    constexpr int TT = 2, NB = 64;
    launch_timed("gate_up_pf", gate_up_pf<TT, NB>, dim3(G * (gs / NB), (T + 64 * TT - 1) / (64 * TT)), dim3(256),
                 s, x, T, d, gs, Wg, Wu, (const int32_t *)ws.tok_list, (const int32_t *)ws.tok_cnt, act);
    down_pf<<<dim3(d / 64, (T + 127) / 128), dim3(256), 0, s>>>(T, d, G, Wd, ws.slot, act, y);
    return hipGetLastError();
}

}  // namespace halo
