// Group-sparse SwiGLU FFN for many tokens (prefill) on the matrix cores, bf16.
//
// With hundreds of tokens the block is a dense contraction per neuron group, but only over
// the tokens that keep the group (paper Sec. II-A: groups are independent until the merge;
// Sec. III-B.3: each token has its own surviving set).  Three kernels:
//
//   group_tokens : for every group, the ascending list of tokens that keep it, and for
//                  every (token, group) the token's slot in that list (-1 = not kept).
//   gate_up_pf   : one workgroup = 32 neurons of one group x up to 256 of the group's
//                  tokens.  The 64 weight rows (32 gate + 32 up) are staged through LDS once
//                  per 64-element K step and shared by the four waves; each wave owns 64
//                  tokens and loads their x rows (gathered by the token list) straight into
//                  registers as the B operand.  Every weight byte is read once from HBM.
//                  act[g][slot][m] = SiLU(gate) * up in bf16.
//   down_pf      : output-stationary: one workgroup = 128 tokens x 64 outputs, walking all
//                  groups; a token that does not keep a group feeds zeros, so it contributes
//                  exactly nothing, and every y element has exactly one writer (no atomics).
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
// gate/up: grid (G * gs/32, ceil(T/256)), 256 threads
// ---------------------------------------------------------------------------
constexpr int kKS = 64;             // K elements per LDS stage
constexpr int kARow = kKS + 8;      // padded LDS row (elements): 144 bytes, conflict-free 16-byte reads

struct BFrags {
    u32x4 v[2][4];                  // [k half of the stage][token tile]
};

__global__ __launch_bounds__(256) void gate_up_pf(
    const bf16_t *__restrict__ x, int T, int d, int gs, const bf16_t *__restrict__ Wg,
    const bf16_t *__restrict__ Wu, const int32_t *__restrict__ tok_list,
    const int32_t *__restrict__ tok_cnt, bf16_t *__restrict__ act)
{
    __shared__ __attribute__((aligned(16))) bf16_t sA[2][64 * kARow];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int i16 = lane & 15, q = lane >> 4;
    const int per_group = gs / 32;
    const int g = blockIdx.x / per_group, nt = blockIdx.x - g * per_group;
    const int cnt = tok_cnt[g];
    const int c0 = blockIdx.y * 256;
    if (c0 >= cnt) return;                                   // uniform for the workgroup
    const int32_t *list = tok_list + (size_t)g * T;
    // this wave's tokens: slots c0 + wave*64 + tt*16 + i16
    const bf16_t *xrow[4];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
        int sl = c0 + wave * 64 + tt * 16 + i16;
        sl = sl < cnt ? sl : cnt - 1;                        // past the end: a valid duplicate, never stored
        xrow[tt] = x + (size_t)list[sl] * d + q * 8;
    }
    // staging role of this thread: row sr (0..31 gate, 32..63 up), 16-byte pieces sp and sp + 4 of 8
    const int sr = tid >> 2, sp = tid & 3;
    const size_t neuron0 = (size_t)g * gs + nt * 32;
    const bf16_t *wsrc = (sr < 32 ? Wg + (neuron0 + sr) * d : Wu + (neuron0 + sr - 32) * d) + sp * 8;
    bf16_t *wdst0 = &sA[0][sr * kARow + sp * 8], *wdst1 = &sA[1][sr * kARow + sp * 8];

    f32x4_t acc[4][4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) acc[mt][tt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    auto load_a = [&](int k0, u32x4 &r0, u32x4 &r1) {
        r0 = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wsrc + k0));
        r1 = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wsrc + k0 + 32));
    };
    auto store_a = [&](bf16_t *dst, const u32x4 &r0, const u32x4 &r1) {
        *reinterpret_cast<u32x4 *>(dst) = r0;
        *reinterpret_cast<u32x4 *>(dst + 32) = r1;
    };
    auto load_b = [&](int k0, BFrags &b) {
#pragma unroll
        for (int kh = 0; kh < 2; ++kh)
#pragma unroll
            for (int tt = 0; tt < 4; ++tt)
                b.v[kh][tt] = *reinterpret_cast<const u32x4 *>(xrow[tt] + k0 + kh * 32);
    };
    auto compute = [&](const bf16_t *a_lds, const BFrags &b) {
#pragma unroll
        for (int kh = 0; kh < 2; ++kh) {
            u32x4 a[4];
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
                a[mt] = *reinterpret_cast<const u32x4 *>(a_lds + (mt * 16 + i16) * kARow + kh * 32 + q * 8);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int tt = 0; tt < 4; ++tt) acc[mt][tt] = mfma16p(a[mt], b.v[kh][tt], acc[mt][tt]);
        }
    };

    // software pipeline over K: while stage s is multiplied, stage s+1's weights travel
    // global -> registers -> the other LDS buffer and its x fragments travel to registers
    const int nstage = d / kKS;                 // even (d % 128 == 0)
    u32x4 ra0, ra1;
    BFrags b0, b1;
    load_a(0, ra0, ra1);
    load_b(0, b0);
    store_a(wdst0, ra0, ra1);
    __syncthreads();
    int s = 0;
    for (; s + 2 < nstage; s += 2) {
        load_a((s + 1) * kKS, ra0, ra1);
        load_b((s + 1) * kKS, b1);
        compute(sA[0], b0);
        store_a(wdst1, ra0, ra1);
        __syncthreads();
        load_a((s + 2) * kKS, ra0, ra1);
        load_b((s + 2) * kKS, b0);
        compute(sA[1], b1);
        store_a(wdst0, ra0, ra1);
        __syncthreads();
    }
    load_a((s + 1) * kKS, ra0, ra1);
    load_b((s + 1) * kKS, b1);
    compute(sA[0], b0);
    store_a(wdst1, ra0, ra1);
    __syncthreads();
    compute(sA[1], b1);

    // D: column = token i16 of tile tt, rows 4q..4q+3 of neuron tile (mt 0,1 = gate; 2,3 = up)
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
        const int sl = c0 + wave * 64 + tt * 16 + i16;
        if (sl < cnt) {
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                uint32_t lo = (uint32_t)f32_to_bf16(silu_mul(acc[mt][tt][0], acc[mt + 2][tt][0])) |
                              ((uint32_t)f32_to_bf16(silu_mul(acc[mt][tt][1], acc[mt + 2][tt][1])) << 16);
                uint32_t hi = (uint32_t)f32_to_bf16(silu_mul(acc[mt][tt][2], acc[mt + 2][tt][2])) |
                              ((uint32_t)f32_to_bf16(silu_mul(acc[mt][tt][3], acc[mt + 2][tt][3])) << 16);
                bf16_t *dst = act + ((size_t)g * T + sl) * gs + nt * 32 + mt * 16 + 4 * q;
                *reinterpret_cast<uint2 *>(dst) = make_uint2(lo, hi);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// down: grid (d/64, ceil(T/128)), 256 threads; each wave 32 tokens x 64 outputs
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void down_pf(
    int T, int d, int G, int gs, const bf16_t *__restrict__ Wd, const int32_t *__restrict__ slot,
    const int32_t *__restrict__ tok_cnt, const bf16_t *__restrict__ act, bf16_t *__restrict__ y)
{
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int i16 = lane & 15, q = lane >> 4;
    const int j0 = blockIdx.x * 64;
    const int t0 = blockIdx.y * 128 + wave * 32;
    if (t0 >= T) return;
    int tok[2];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
        const int t = t0 + tt * 16 + i16;
        tok[tt] = t < T ? t : T - 1;                         // duplicate of a valid token, never stored
    }
    f32x4_t acc[4][2];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) acc[mt][tt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const int ksteps = gs / 32;
    const u32x4 zero = {0u, 0u, 0u, 0u};
    for (int g = 0; g < G; ++g) {
        if (tok_cnt[g] == 0) continue;                       // uniform
        const int s0 = slot[(size_t)tok[0] * G + g], s1 = slot[(size_t)tok[1] * G + g];
        const bf16_t *pb0 = act + ((size_t)g * T + (s0 < 0 ? 0 : s0)) * gs + q * 8;
        const bf16_t *pb1 = act + ((size_t)g * T + (s1 < 0 ? 0 : s1)) * gs + q * 8;
        const bf16_t *pa = Wd + ((size_t)g * d + j0 + i16) * gs + q * 8;
        for (int ks = 0; ks < ksteps; ++ks) {
            u32x4 a[4];
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
                a[mt] = *reinterpret_cast<const u32x4 *>(pa + (size_t)mt * 16 * gs + ks * 32);
            const u32x4 b0 = s0 < 0 ? zero : *reinterpret_cast<const u32x4 *>(pb0 + ks * 32);
            const u32x4 b1 = s1 < 0 ? zero : *reinterpret_cast<const u32x4 *>(pb1 + ks * 32);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
                acc[mt][0] = mfma16p(a[mt], b0, acc[mt][0]);
                acc[mt][1] = mfma16p(a[mt], b1, acc[mt][1]);
            }
        }
    }
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
    return T > 1 && d % 128 == 0 && gs % 32 == 0;
}

hipError_t launch_ffn_prefill(const bf16_t *x, int T, int d, int G, int gs, const bf16_t *Wg,
                              const bf16_t *Wu, const bf16_t *Wd, const uint8_t *mask, bf16_t *y,
                              const DecodeScratch &ws, hipStream_t s)
{
    bf16_t *act = reinterpret_cast<bf16_t *>(ws.act);
    group_tokens_kernel<<<dim3(G), dim3(256), 0, s>>>(mask, T, G, ws.tok_list, ws.tok_cnt, ws.slot);
    launch_timed("gate_up_pf", gate_up_pf, dim3(G * (gs / 32), (T + 255) / 256), dim3(256), s, x, T, d, gs, Wg,
                 Wu, (const int32_t *)ws.tok_list, (const int32_t *)ws.tok_cnt, act);
    down_pf<<<dim3(d / 64, (T + 127) / 128), dim3(256), 0, s>>>(T, d, G, gs, Wd, ws.slot, ws.tok_cnt, act, y);
    return hipGetLastError();
}

}  // namespace halo
