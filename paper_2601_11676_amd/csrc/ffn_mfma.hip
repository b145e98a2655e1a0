// Group-sparse SwiGLU FFN for a few tokens (2 <= T <= 16) on the matrix cores, bf16.
//
// The block is still bound by streaming the surviving groups' weights from HBM (every
// weight byte is used T times), so the layout of the work follows the memory stream and
// the matrix instruction is only a cheap way to apply one 16-byte weight piece to all
// tokens at once (v_mfma_f32_16x16x32_bf16: 16 weight rows x 16 tokens x 32 elements).
//
//   gate/up : each wave owns a contiguous run of the union's neurons (runs differ by at
//             most one), cut into tiles of <= 16 rows; a lane loads 64 contiguous bytes of
//             its row per step; the token fragments come from an LDS copy of x.
//             act[t][n] = mask ? SiLU(gate)*up : 0 is stored in bf16.
//   down    : Wd is group-blocked, Wd[g][j][m]; a workgroup owns 16 output rows j, its four
//             waves split the union's groups, partial tiles are added through LDS and y is
//             written directly.
// Operand layout of the instruction (wave64): A lane l holds row l%16, elements
// 8*(l/16)..+7 of the 32; B lane l holds column l%16, same elements; D lane l holds
// column l%16, rows 4*(l/16)..+3.  Rows are neurons (or outputs j), columns are tokens.
#include "kernels.hpp"

namespace halo {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4_t mfma16(const u32x4 &a, const u32x4 &b, const f32x4_t &c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

constexpr int kXPad = 8;   // bf16 elements of padding per LDS row of x: rows start 16 bytes apart in bank space

// grid: any number of 256-thread workgroups; dynamic LDS = T * (d + kXPad) * 2 bytes
__global__ __launch_bounds__(256) void gate_up_mt(
    const bf16_t *__restrict__ x, int T, int d, int G, int gs, const bf16_t *__restrict__ Wg,
    const bf16_t *__restrict__ Wu, const uint8_t *__restrict__ mask, const int32_t *__restrict__ ulist,
    const int32_t *__restrict__ meta, bf16_t *__restrict__ act, int act_stride)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *xl = reinterpret_cast<bf16_t *>(smem);
    const int xs = d + kXPad;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int pieces = d / 8;
    for (int idx = tid; idx < T * pieces; idx += 256) {
        const int t = idx / pieces, c = idx - t * pieces;
        *reinterpret_cast<u32x4 *>(xl + (size_t)t * xs + c * 8) =
            *reinterpret_cast<const u32x4 *>(x + (size_t)t * d + c * 8);
    }
    __syncthreads();
    const long long total = (long long)meta[0] * gs;
    const int nw = gridDim.x * 4, w = blockIdx.x * 4 + wave;
    const int n0 = (int)(total * w / nw), n1 = (int)(total * (w + 1) / nw);
    const int L = n1 - n0;
    if (L <= 0) return;
    const int ntile = (L + 15) / 16;
    const int i = lane & 15, q = lane >> 4;
    const int tok = i < T ? i : T - 1;                      // columns >= T repeat the last token, unused
    const bf16_t *xrow = xl + (size_t)tok * xs + q * 32;
    for (int tile = 0; tile < ntile; ++tile) {
        const int r0 = n0 + (int)((long long)L * tile / ntile);
        const int r1 = n0 + (int)((long long)L * (tile + 1) / ntile);     // r1 - r0 <= 16
        const int n = r0 + i < r1 ? r0 + i : r1 - 1;       // rows past the tile repeat its last row
        const int u = n / gs;
        const size_t wrow = (size_t)ulist[u] * gs + (n - u * gs);
        const bf16_t *pg = Wg + wrow * d + q * 32;
        const bf16_t *pu = Wu + wrow * d + q * 32;
        f32x4_t cg = {0.f, 0.f, 0.f, 0.f}, cu = {0.f, 0.f, 0.f, 0.f};
        // 256 elements of every row per step: sixteen 16-byte loads in flight per lane
        int ks = 0;
        for (; ks + 256 <= d; ks += 256) {
            u32x4 ag[8], au[8], b[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int off = ks + (j >> 2) * 128 + (j & 3) * 8;
                ag[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(pg + off));
                au[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(pu + off));
            }
#pragma unroll
            for (int j = 0; j < 8; ++j)
                b[j] = *reinterpret_cast<const u32x4 *>(xrow + ks + (j >> 2) * 128 + (j & 3) * 8);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                cg = mfma16(ag[j], b[j], cg);
                cu = mfma16(au[j], b[j], cu);
            }
        }
        for (; ks < d; ks += 128) {
            u32x4 ag[4], au[4], b[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                ag[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(pg + ks + j * 8));
                au[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(pu + ks + j * 8));
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = *reinterpret_cast<const u32x4 *>(xrow + ks + j * 8);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                cg = mfma16(ag[j], b[j], cg);
                cu = mfma16(au[j], b[j], cu);
            }
        }
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

// grid: d/16 workgroups of 256 threads; gs % 32 == 0
constexpr int kDownGroups = 4;     // groups in flight per wave

__global__ __launch_bounds__(256) void down_mt(
    int T, int d, int gs, const bf16_t *__restrict__ Wd, const int32_t *__restrict__ ulist,
    const int32_t *__restrict__ meta, const bf16_t *__restrict__ act, int act_stride,
    bf16_t *__restrict__ y)
{
    __shared__ float red[4][64][4];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int i = lane & 15, q = lane >> 4;
    const int j0 = blockIdx.x * 16;
    const int n_u = meta[0];
    const int u0 = n_u * wave / 4, u1 = n_u * (wave + 1) / 4;
    const int tok = i < T ? i : T - 1;
    const int ksteps = gs / 32;
    const bf16_t *arow = act + (size_t)tok * act_stride + q * 8;
    const size_t gstride = (size_t)d * gs;
    const bf16_t *wrow = Wd + (size_t)(j0 + i) * gs + q * 8;
    f32x4_t c = {0.f, 0.f, 0.f, 0.f};
    if (ksteps == 4) {
        for (int ub = u0; ub < u1; ub += kDownGroups) {
            u32x4 a[kDownGroups][4], b[kDownGroups][4];
#pragma unroll
            for (int k = 0; k < kDownGroups; ++k) {
                const int u = ub + k < u1 ? ub + k : ub;           // past the end: in-range duplicate
                const bf16_t *pw = wrow + ulist[u] * gstride;
                const bf16_t *pa = arow + (size_t)u * gs;
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    a[k][s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(pw + s * 32));
                    b[k][s] = *reinterpret_cast<const u32x4 *>(pa + s * 32);
                }
            }
#pragma unroll
            for (int k = 0; k < kDownGroups; ++k) {
                if (ub + k < u1) {
#pragma unroll
                    for (int s = 0; s < 4; ++s) c = mfma16(a[k][s], b[k][s], c);
                }
            }
        }
    } else {
        for (int u = u0; u < u1; ++u) {
            const bf16_t *pw = wrow + ulist[u] * gstride;
            const bf16_t *pa = arow + (size_t)u * gs;
            for (int s = 0; s < ksteps; ++s) {
                const u32x4 a = *reinterpret_cast<const u32x4 *>(pw + s * 32);
                const u32x4 b = *reinterpret_cast<const u32x4 *>(pa + s * 32);
                c = mfma16(a, b, c);
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

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
static int max_lds_bytes()
{
    static int cached = -1;
    if (cached < 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess)
            v = 65536;
        cached = v;
    }
    return cached;
}

bool mfma_path_supported(int T, int d, int gs)
{
    if (T < 2 || T > 16 || d % 128 != 0 || gs % 32 != 0) return false;
    return (long long)T * (d + kXPad) * 2 <= max_lds_bytes();
}

hipError_t launch_ffn_mfma(const bf16_t *x, int T, int d, int G, int gs, const bf16_t *Wg,
                           const bf16_t *Wu, const bf16_t *Wd, const uint8_t *mask, bf16_t *y,
                           const DecodeScratch &ws, hipStream_t s)
{
    const int ffn = G * gs;
    bf16_t *act = reinterpret_cast<bf16_t *>(ws.act);
    hipError_t e = launch_union(mask, T, G, ws.ulist, ws.meta, s);
    if (e != hipSuccess) return e;
    const size_t lds = (size_t)T * (d + kXPad) * 2;
    static size_t lds_enabled = 0;
    if (lds > 65536 && lds > lds_enabled) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(gate_up_mt),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        lds_enabled = lds;
    }
    launch_timed_lds("gate_up_mt", gate_up_mt, dim3(256), dim3(256), lds, s, x, T, d, G, gs, Wg, Wu, mask,
                     (const int32_t *)ws.ulist, (const int32_t *)ws.meta, act, ffn);
    down_mt<<<dim3(d / 16), dim3(256), 0, s>>>(T, d, gs, Wd, ws.ulist, ws.meta, act, ffn, y);
    return hipGetLastError();
}

}  // namespace halo
