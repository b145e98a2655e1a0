// Group-sparse SwiGLU FFN for many tokens (prefill) on the matrix cores, bf16.
//
// With hundreds of tokens the block is a dense contraction per neuron group, but only over
// the tokens that keep the group (paper Sec. II-A: groups are independent until the merge;
// Sec. III-B.3: each token has its own surviving set).  Kernels:
//
//   group_tokens : for every group, the ascending list of tokens that keep it, and for
//                  every (token, group) the token's slot in that list (-1 = not kept); also
//                  keeps one zero row per group in the activation buffer.
//   gate_up_pf_ring : one workgroup = 64 neurons of one group (64 gate + 64 up rows) x up to 256
//                  of the group's tokens (x rows gathered by the token list); both operands
//                  travel straight from memory into a ring of K stages in LDS.
//                  act[g][slot][m] = SiLU(gate) * up in bf16.
//   down_pf_ring : one workgroup = 128 outputs x 256 tokens over a range of groups, same ring;
//                  a token that does not keep a group reads the group's zero row, so it
//                  contributes exactly nothing.  With several ranges the fp32 partial sums are
//                  added by reduce_partials in fixed order; every element has one writer.
//   down_pf      : the earlier output-stationary form (128 tokens x 64 outputs per workgroup,
//                  walking all groups), kept for shapes the ring form does not take (more
//                  than 256 groups, more than 32767 tokens).
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
                                                           int32_t *__restrict__ slot, bf16_t *__restrict__ act)
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
    // the row after the group's last activation row is kept zero (group size 128): the down
    // projection points the tokens that do not keep the group at it
    const int cnt = s_base;
    if (cnt < T && tid < 64) reinterpret_cast<uint32_t *>(act + ((size_t)g * T + cnt) * 128)[tid] = 0u;
}

// ---------------------------------------------------------------------------
// gate/up through rings in LDS filled by direct global -> LDS loads
// grid: 8 * ceil(items / 8) workgroups of 256 threads, 144 KiB of dynamic LDS, one per compute unit
// ---------------------------------------------------------------------------
// Workgroup tile: 128 weight rows (64 gate + 64 up neurons of one group) x 256 of the group's
// tokens; K advances 64 elements per stage.  In LDS a stage is 128 weight rows and 256 gathered x
// rows of 128 bytes.  One load instruction moves 1 KiB = 8 rows x 128 bytes, lane l landing at byte
// 16 l of the block; to keep the operand reads free of bank conflicts the 16-byte piece p of tile row
// r is parked at position p ^ (r & 7) of its row, which the loading lane arranges by fetching piece
// (l & 7) ^ (l >> 3).  Nothing passes through registers on the way.
//
// A stage is 48 KiB and a ring holds three, so a stage is requested three steps before the matrix
// instructions use it.  Each wave fetches a quarter of every stage (4 blocks of weight rows, 8 blocks
// of x rows).  Lanes whose token row lies past the end of the group's list are switched off for the
// load (lane 0 stays on, so that the load counts as one of the wave's outstanding loads whatever the
// hardware does with an empty one): the number of loads per stage stays fixed and nothing is moved
// for rows that do not exist.
//
// For the matrix work the four waves are a 2 x 2 grid: two halves of the stage's K range (elements
// 0..31 / 32..63) times two halves of the token tile, so a wave owns a 128 x 128 partial tile (256
// accumulator registers) and reads 16 KiB of LDS per 64 matrix instructions; the two K halves are
// added through LDS once at the end.
constexpr int kRingTok = 256;
constexpr int kRingStages = 3;
constexpr int kRingStageBytes = (128 + kRingTok) * 128;          // 48 KiB: weight rows, then x rows
constexpr int kRingBytes = kRingStages * kRingStageBytes;        // 144 KiB (the final exchange needs 128 KiB)

// One direct global -> LDS load of 16 bytes per lane: lane l's bytes at base + offset land at LDS
// address lds_addr + 16 l (m0 carries the LDS address).  Done only if the wave-uniform `cond` holds,
// and only for the lanes of `lanes` (all 64 lanes of the wave are active around it).  The branch is
// inside the statement on purpose: a branch the compiler can see splits the step into basic blocks,
// and it then shuffles the accumulators between register files at the joins.
// STREAM: the bytes are used once by this die (weight rows): the load carries the non-temporal hint, so
// that they do not push the rows that are used again (x, act) out of the die's L2.
template <bool STREAM = false>
__device__ __forceinline__ void load_to_lds16_if(bool cond, unsigned long long lanes, const void *base,
                                                 uint32_t offset, uint32_t lds_addr)
{
    unsigned long long saved_exec;       // the lanes active around the statement come back afterwards
    if (STREAM)
        asm volatile("s_cmp_eq_u32 %4, 0\n\ts_cbranch_scc1 1f\n\ts_mov_b32 m0, %3\n\ts_mov_b64 %0, exec\n\t"
                     "s_mov_b64 exec, %5\n\tglobal_load_lds_dwordx4 %1, %2 nt\n\ts_mov_b64 exec, %0\n1:"
                     : "=&s"(saved_exec)
                     : "v"(offset), "s"(base), "s"(lds_addr), "s"(__builtin_amdgcn_readfirstlane((uint32_t)cond)),
                       "s"(lanes)
                     : "memory", "scc");    // m0 is reserved: the compiler sets it anew before each use of its own
    else
        asm volatile("s_cmp_eq_u32 %4, 0\n\ts_cbranch_scc1 1f\n\ts_mov_b32 m0, %3\n\ts_mov_b64 %0, exec\n\t"
                     "s_mov_b64 exec, %5\n\tglobal_load_lds_dwordx4 %1, %2\n\ts_mov_b64 exec, %0\n1:"
                     : "=&s"(saved_exec)
                     : "v"(offset), "s"(base), "s"(lds_addr), "s"(__builtin_amdgcn_readfirstlane((uint32_t)cond)),
                       "s"(lanes)
                     : "memory", "scc");
}

// wait until at most N (deep) or none of the wave's loads are outstanding
template <int N>
__device__ __forceinline__ void wait_loads(bool deep)
{
    asm volatile("s_cmp_eq_u32 %0, 0\n\ts_cbranch_scc1 1f\n\ts_waitcnt vmcnt(%1)\n\ts_branch 2f\n1:\n\t"
                 "s_waitcnt vmcnt(0)\n2:" ::"s"(__builtin_amdgcn_readfirstlane((uint32_t)deep)),
                 "n"(N)
                 : "memory", "scc");
}

// acc += a * b with the accumulator pinned to the accumulation registers and updated in place.
// (Left to itself the compiler gives the 64 tiles of this kernel rotating destination registers and
// moves a few hundred registers between the two files per step to make that work.)  A statement the
// compiler cannot look into also gets none of its matrix-pipeline wait states, which is safe here:
// a tile is touched again 63 matrix instructions later (a 16x16x32 bf16 instruction occupies the
// pipeline for 8 passes of 4 cycles, so its result is long written back by then), and the first
// ordinary read of the accumulators comes after a barrier and an explicit pause of 2 x 16 idle
// cycles, more than the 18 cycles the last instruction can still be in flight.
__device__ __forceinline__ void mfma16_inplace(f32x4_t &acc, const u32x4 &a, const u32x4 &b)
{
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

// Token tiles are numbered group by group (group g has ceil(cnt[g] / tile_tokens) of them), and only
// tiles that exist get a number, so the working workgroups are consecutive.  Called by whole waves;
// results are the same in every lane.
__device__ __forceinline__ int wave_inclusive_sum(int n, int lane)
{
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int v = __shfl_up(n, off);
        if (lane >= off) n += v;
    }
    return n;
}

__device__ __forceinline__ int count_tiles(const int32_t *__restrict__ tok_cnt, int G, int tile_tokens, int lane)
{
    int total = 0;
    for (int g0 = 0; g0 < G; g0 += 64) {
        const int g = g0 + lane;
        const int n = g < G ? (tok_cnt[g] + tile_tokens - 1) / tile_tokens : 0;
        total += __shfl(wave_inclusive_sum(n, lane), 63);
    }
    return total;
}

// group and tile within the group of tile number `target` (< count_tiles)
__device__ __forceinline__ int2 find_tile(const int32_t *__restrict__ tok_cnt, int G, int tile_tokens, int target,
                                          int lane)
{
    int base = 0;
    for (int g0 = 0; g0 < G; g0 += 64) {
        const int g = g0 + lane;
        const int n = g < G ? (tok_cnt[g] + tile_tokens - 1) / tile_tokens : 0;
        const int incl = wave_inclusive_sum(n, lane);
        const int total = __shfl(incl, 63);
        if (target < base + total) {
            const unsigned long long m = __ballot(target < base + incl);
            const int l = __ffsll((long long)m) - 1;
            const int excl = __shfl(incl - n, l);
            return make_int2(g0 + l, target - base - excl);
        }
        base += total;
    }
    return make_int2(-1, 0);
}

struct RingFrags {
    u32x4 a[8], b[8];
};

template <int KS_HALF>
__device__ __forceinline__ void ring_finish(f32x4_t (&acc)[8][8], unsigned char *ring, int wave, int lane,
                                            bool active, bf16_t *__restrict__ act_row0, int sl0, int cnt)
{
    // the wave keeps token tiles 4 KS_HALF .. +3 and hands the other four to its partner (wave ^ 1)
    constexpr int own = 4 * KS_HALF, other = 4 - own;
    if (active) {
        unsigned char *mine = ring + wave * 32768 + lane * 16;
#pragma unroll
        for (int mt = 0; mt < 8; ++mt)
#pragma unroll
            for (int j = 0; j < 4; ++j) *reinterpret_cast<f32x4_t *>(mine + (mt * 4 + j) * 1024) = acc[mt][other + j];
    }
    __syncthreads();
    if (!active) return;
    const unsigned char *theirs = ring + (wave ^ 1) * 32768 + lane * 16;
    const int i16 = lane & 15, q = lane >> 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int sl = sl0 + (own + j) * 16 + i16;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
            const f32x4_t g = acc[mt][own + j] + *reinterpret_cast<const f32x4_t *>(theirs + (mt * 4 + j) * 1024);
            const f32x4_t u = acc[mt + 4][own + j] + *reinterpret_cast<const f32x4_t *>(theirs + ((mt + 4) * 4 + j) * 1024);
            const uint32_t lo = (uint32_t)f32_to_bf16(silu_mul_fast(g[0], u[0])) | ((uint32_t)f32_to_bf16(silu_mul_fast(g[1], u[1])) << 16);
            const uint32_t hi = (uint32_t)f32_to_bf16(silu_mul_fast(g[2], u[2])) | ((uint32_t)f32_to_bf16(silu_mul_fast(g[3], u[3])) << 16);
            if (sl < cnt) *reinterpret_cast<uint2 *>(act_row0 + (size_t)sl * 128 + mt * 16 + 4 * q) = make_uint2(lo, hi);
        }
    }
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void gate_up_pf_ring(
    const bf16_t *__restrict__ x, int T, int d, int G, const bf16_t *__restrict__ Wg, const bf16_t *__restrict__ Wu,
    const int32_t *__restrict__ tok_list, const int32_t *__restrict__ tok_cnt, bf16_t *__restrict__ act)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char ring[];
    constexpr int gs = 128;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ks = wave & 1, nh = wave >> 1;
    const int i16 = lane & 15, q = lane >> 4;
    // Workgroups are dealt to the eight dies round-robin by their index.  The work items (tile, half
    // of the group's neurons) are numbered so that a die gets a consecutive run of them: the two
    // halves of a tile share their x rows, the tiles of a group share its weight rows, and all
    // workgroups of a die walk K from the same starting stage, so those rows are found in the die's
    // own L2.  Numbering only the tiles that exist also spreads the work evenly over the dies (with
    // a (group, chunk) grid the empty chunks left some dies with more workgroups than compute units).
    const int n_items = 2 * count_tiles(tok_cnt, G, kRingTok, lane);
    const int per_die = (n_items + 7) >> 3;
    const int die = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int item = __builtin_amdgcn_readfirstlane(die * per_die + slot);
    if (slot >= per_die || item >= n_items) return;              // uniform for the workgroup
    const int nt = item & 1;
    const int2 tile = find_tile(tok_cnt, G, kRingTok, item >> 1, lane);
    const int g = __builtin_amdgcn_readfirstlane(tile.x);
    const int cnt = tok_cnt[g];
    const int c0 = __builtin_amdgcn_readfirstlane(tile.y) * kRingTok;
    const int32_t *list = tok_list + (size_t)g * T;
    const bool active = c0 + nh * 128 < cnt;                     // this wave's half of the tile holds tokens

    // The dies start at different K stages (rows are a power of two apart: with everybody at the same
    // K offset all requests of a moment would go to the same few memory channels).
    const int ns = d / 64;                                       // even, >= 2
    int kstage = (die * ns) >> 3;                                // stage of the next request
    // loading role: the stage's 48 blocks of 8 rows are dealt round-robin, wave w takes blocks w + 4 j:
    // j = 0, 1 gate rows, j = 2, 3 up rows, then j = 0..7 of the x rows
    const int br = lane >> 3;
    const int piece = (lane & 7) ^ br;
    const bf16_t *src_g = Wg + ((size_t)g * gs + nt * 64) * d + kstage * 64;
    const bf16_t *src_u = Wu + ((size_t)g * gs + nt * 64) * d + kstage * 64;
    const bf16_t *src_x = x + kstage * 64;
    uint32_t off_w[4], off_x[8];                                 // byte offset of the lane's piece of block j
    unsigned long long lanes_x[8];                               // lanes whose token row exists
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = (wave + 4 * (j & 1)) * 8 + br;             // 0..63 within the gate or the up half
        off_w[j] = (uint32_t)(r * d + piece * 8) * 2u;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int sl = c0 + (wave + 4 * j) * 8 + br;
        lanes_x[j] = __ballot(sl < cnt) | 1ull;
        off_x[j] = (uint32_t)(list[sl < cnt ? sl : cnt - 1] * d + piece * 8) * 2u;
    }
    const uint32_t wdst0 = (uint32_t)(size_t)ring + wave * 1024; // this wave's first block of stage buffer 0
    auto advance = [&](bool yes) {                               // on to the next stage, with wrap-around
        const bool wrap = kstage + 1 == ns;
        const int delta = yes ? (wrap ? 64 - d : 64) : 0;
        src_g += delta;
        src_u += delta;
        src_x += delta;
        kstage = yes ? (wrap ? 0 : kstage + 1) : kstage;
    };
    // operand reads: tile row mt*16 + i16 (or token row), piece (4 ks + q) at its swizzled position
    const int loff = i16 * 128 + (((4 * ks + q) ^ (i16 & 7)) * 16);
    f32x4_t acc[8][8];
#pragma unroll
    for (int mt = 0; mt < 8; ++mt)
#pragma unroll
        for (int tt = 0; tt < 8; ++tt) acc[mt][tt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // Stage s lives in ring buffer s % 3.  At the top of step s the fragments of stage s are in
    // registers.  The barrier of step s says: everybody's part of stage s+1 has landed and everybody
    // has finished reading stage s, whose buffer is then handed to stage s+3.  The matrix work of a
    // step is cut into eight slices of eight instructions (one 16-row tile of the weights against the
    // eight token tiles) with one or two of the step's twelve loads in front of each: a wave issues in
    // order, and a burst of memory instructions fills the memory pipelines' queues and holds the
    // matrix instructions behind it back for as long as the burst takes to drain.
    // (Waves whose half of the token tile is empty run the matrix work all the same, on whatever the
    // x buffer holds: they sit on a SIMD of their own and nothing they compute is stored.)
    for (int i = 0; i < kRingStages && i < ns; ++i) {
        const uint32_t dst = wdst0 + i * kRingStageBytes;
#pragma unroll
        for (int j = 0; j < 4; ++j) load_to_lds16_if<true>(true, ~0ull, j < 2 ? src_g : src_u, off_w[j], dst + j * 4096);
#pragma unroll
        for (int j = 0; j < 8; ++j) load_to_lds16_if(true, lanes_x[j], src_x, off_x[j], dst + 16384 + j * 4096);
        advance(true);
    }
    wait_loads<24>(ns >= kRingStages);
    __syncthreads();
    RingFrags F0, F1;
    {
        const unsigned char *pa = ring + loff, *px = ring + 16384 + nh * 16384 + loff;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            F0.a[c] = *reinterpret_cast<const u32x4 *>(pa + c * 2048);
            F0.b[c] = *reinterpret_cast<const u32x4 *>(px + c * 2048);
        }
    }
    int buf = 0;                                                 // buffer of stage s
    auto step = [&](const RingFrags &cur, RingFrags &next, int s) __attribute__((always_inline)) {
        const int nbuf = buf == kRingStages - 1 ? 0 : buf + 1;
        wait_loads<12>(s + kRingStages <= ns);                   // stage s+2 may still be on its way
        __syncthreads();
        const bool go = s + kRingStages < ns;
        const uint32_t dst = wdst0 + buf * kRingStageBytes;
        __builtin_amdgcn_sched_barrier(0);
        {   // (in the last step this reads a stage that does not exist: in bounds, unused)
            const unsigned char *pa = ring + nbuf * kRingStageBytes + loff;
            const unsigned char *px = pa + 16384 + nh * 16384;
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                next.a[c] = *reinterpret_cast<const u32x4 *>(pa + c * 2048);
                next.b[c] = *reinterpret_cast<const u32x4 *>(px + c * 2048);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            load_to_lds16_if(go, lanes_x[c], src_x, off_x[c], dst + 16384 + c * 4096);
            if (c < 4) load_to_lds16_if<true>(go, ~0ull, c < 2 ? src_g : src_u, off_w[c], dst + c * 4096);
#pragma unroll
            for (int tt = 0; tt < 8; ++tt) mfma16_inplace(acc[c][tt], cur.a[c], cur.b[tt]);
            __builtin_amdgcn_sched_barrier(0);
        }
        advance(go);
        buf = nbuf;
    };
    for (int s = 0; s < ns; s += 2) {
        step(F0, F1, s);
        step(F1, F0, s + 1);
    }
    __syncthreads();                                             // every wave is done with the rings
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");           // the last matrix results are in the registers

    bf16_t *act_row0 = act + (size_t)g * T * gs + nt * 64;
    const int sl0 = c0 + nh * 128;
    if (ks == 0)
        ring_finish<0>(acc, ring, wave, lane, active, act_row0, sl0, cnt);
    else
        ring_finish<1>(acc, ring, wave, lane, active, act_row0, sl0, cnt);
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
// down projection through the same kind of ring, groups split over workgroups
// grid: 8 * ceil(items / 8) workgroups of 256 threads, 160 KiB of dynamic LDS
// ---------------------------------------------------------------------------
// Workgroup tile: 128 outputs x 256 tokens, over a contiguous range of the groups (the K
// dimension): with 128 x 256 tiles alone a 512-token call would occupy 64 compute units, so the
// groups are cut into `splits` ranges and every range goes to its own workgroup, which leaves its
// fp32 partial sums in partial[split][t][j]; reduce_partials adds the ranges in fixed order.  With a
// single range the workgroup writes y itself.
//
// A stage is half a group (64 of its 128 neurons): 128 rows of Wd (the group's 128 x 128 tile is 32
// KiB of consecutive bytes, a stage takes alternate halves of its 256-byte rows) and the 256 token
// rows of act, found through the slot table.  A token that does not keep the group is pointed at
// the group's row of zeros (row cnt[g], written by group_tokens), so it contributes exactly nothing.
// The row indices of the workgroup's tokens for all its groups are put into LDS once, 16 bits each.
// Everything else is as in gate_up_pf_ring.
constexpr int kDownSlotBytes = 160 * 1024 - kRingBytes;          // 16 KiB: 32 groups x 256 tokens x 2 bytes
constexpr int kDownMaxGroups = kDownSlotBytes / (kRingTok * 2);
constexpr int kDownMaxSplits = 8;

// number of group ranges for the ring kernel, 0 = shape not covered by it
int prefill_down_splits(int T, int d, int G)
{
    if (d % 128 != 0 || T > 32767) return 0;
    const int tiles = (d / 128) * ((T + kRingTok - 1) / kRingTok);
    int splits = (256 + tiles / 2) / tiles;                      // about one workgroup per compute unit
    const int need = (G + kDownMaxGroups - 1) / kDownMaxGroups;  // the slot table must fit
    splits = splits < need ? need : splits;
    splits = splits < 1 ? 1 : splits;
    splits = splits > G ? G : splits;
    if (splits > kDownMaxSplits || (G + splits - 1) / splits > kDownMaxGroups) return 0;
    return splits;
}

template <int KS_HALF>
__device__ __forceinline__ void down_finish(f32x4_t (&acc)[8][8], unsigned char *ring, int wave, int lane, int t0,
                                            int T, int d, int j0, float *__restrict__ partial, bf16_t *__restrict__ y)
{
    // the wave keeps token tiles 4 KS_HALF .. +3 and hands the other four to its partner (wave ^ 1)
    constexpr int own = 4 * KS_HALF, other = 4 - own;
    unsigned char *mine = ring + wave * 32768 + lane * 16;
#pragma unroll
    for (int mt = 0; mt < 8; ++mt)
#pragma unroll
        for (int j = 0; j < 4; ++j) *reinterpret_cast<f32x4_t *>(mine + (mt * 4 + j) * 1024) = acc[mt][other + j];
    __syncthreads();
    const unsigned char *theirs = ring + (wave ^ 1) * 32768 + lane * 16;
    const int i16 = lane & 15, q = lane >> 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int t = t0 + (own + j) * 16 + i16;
#pragma unroll
        for (int mt = 0; mt < 8; ++mt) {
            const f32x4_t v = acc[mt][own + j] + *reinterpret_cast<const f32x4_t *>(theirs + (mt * 4 + j) * 1024);
            if (t < T) {
                const size_t at = (size_t)t * d + j0 + mt * 16 + 4 * q;
                if (partial) {
                    *reinterpret_cast<f32x4_t *>(partial + at) = v;
                } else {
                    const uint32_t lo = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
                    const uint32_t hi = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
                    *reinterpret_cast<uint2 *>(y + at) = make_uint2(lo, hi);
                }
            }
        }
    }
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void down_pf_ring(
    int T, int d, int G, int splits, const bf16_t *__restrict__ Wd, const int32_t *__restrict__ slot,
    const int32_t *__restrict__ tok_cnt, const bf16_t *__restrict__ act, float *__restrict__ partial,
    bf16_t *__restrict__ y)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char ring[];
    int16_t *s_row = reinterpret_cast<int16_t *>(ring + kRingBytes);    // [group of the range][token of the tile]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ks = wave & 1, nh = wave >> 1;
    const int i16 = lane & 15, q = lane >> 4;
    // work items: (token tile, group range, output tile) triples; a die gets a consecutive run of them
    const int n_ot = d / 128;
    const int n_items = n_ot * ((T + kRingTok - 1) / kRingTok) * splits;
    const int per_die = (n_items + 7) >> 3;
    const int die = blockIdx.x & 7, dslot = blockIdx.x >> 3;
    const int item = die * per_die + dslot;
    if (dslot >= per_die || item >= n_items) return;             // uniform for the workgroup
    // Two numberings.  With one or two token tiles the items of a die are the token tiles of consecutive
    // output tiles of one range: a tile of Wd is fetched from memory by the first and found in the die's
    // L2 by the second, and the act rows of both token tiles fit beside it.  With more token tiles the
    // items of a die share one token tile's act rows instead (they would not all fit).
    const int n_tt = (T + kRingTok - 1) / kRingTok;
    int ttile, split, j0;
    if (n_tt <= 2) {
        ttile = item % n_tt;
        const int rest = item / n_tt;
        split = rest / n_ot;
        j0 = (rest - split * n_ot) * 128;
    } else {
        const int pair = item / n_ot;
        j0 = (item - pair * n_ot) * 128;
        ttile = pair / splits;
        split = pair - ttile * splits;
    }
    const int t0 = ttile * kRingTok;
    const int g_lo = (int)((long long)split * G / splits), g_hi = (int)((long long)(split + 1) * G / splits);
    const int ng = g_hi - g_lo;                                  // >= 1, <= kDownMaxGroups
    const int ns = 2 * ng;

    // rows of act for this thread's token and every group of the range
    {
        // eight groups' slots and counts are requested together: one memory round trip per eight groups,
        // not two per group
        const int t = t0 + tid;
        const int32_t *my = slot + (size_t)(t < T ? t : T - 1) * G + g_lo;
        for (int gi0 = 0; gi0 < ng; gi0 += 8) {
            int row[8], zero_row[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int gi = gi0 + k < ng ? gi0 + k : ng - 1;
                row[k] = my[gi];
                zero_row[k] = tok_cnt[g_lo + gi];                // the group's row of zeros
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                // (a token past the end: any row, never stored)
                if (gi0 + k < ng) s_row[(gi0 + k) * kRingTok + tid] = (int16_t)(t < T ? (row[k] < 0 ? zero_row[k] : row[k]) : 0);
            }
        }
    }
    __syncthreads();

    // loading role: the stage's 48 blocks of 8 rows are dealt round-robin, wave w takes blocks w + 4 j:
    // j = 0..3 of the Wd rows, j = 0..7 of the act rows
    const int br = lane >> 3;
    const int piece = (lane & 7) ^ br;
    const bf16_t *src_w = Wd + ((size_t)g_lo * d + j0) * 128;    // the stage's Wd half rows; + 64 elements for odd stages
    const bf16_t *src_a = act + (size_t)g_lo * T * 128;
    uint32_t off_w[4], off_a[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) off_w[j] = (uint32_t)(((wave + 4 * j) * 8 + br) * 128 + piece * 8) * 2u;
    auto rows_of_group = [&](int gi) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            off_a[j] = (uint32_t)(s_row[gi * kRingTok + (wave + 4 * j) * 8 + br] * 128 + piece * 8) * 2u;
    };
    const uint32_t wdst0 = (uint32_t)(size_t)ring + wave * 1024;
    int next_stage = 0;                                          // stage of the next request
    auto advance = [&](bool yes) {
        const bool odd = next_stage & 1;
        src_w += yes ? (odd ? (ptrdiff_t)d * 128 - 64 : 64) : 0;
        src_a += yes ? (odd ? (ptrdiff_t)T * 128 - 64 : 64) : 0;
        next_stage += yes ? 1 : 0;
    };
    const int loff = i16 * 128 + (((4 * ks + q) ^ (i16 & 7)) * 16);
    f32x4_t acc[8][8];
#pragma unroll
    for (int mt = 0; mt < 8; ++mt)
#pragma unroll
        for (int tt = 0; tt < 8; ++tt) acc[mt][tt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    rows_of_group(0);
    for (int i = 0; i < kRingStages && i < ns; ++i) {
        if (i == 2) rows_of_group(1);                            // ns > 2: a second group exists
        const uint32_t dst = wdst0 + i * kRingStageBytes;
#pragma unroll
        for (int j = 0; j < 4; ++j) load_to_lds16_if(true, ~0ull, src_w, off_w[j], dst + j * 4096);
#pragma unroll
        for (int j = 0; j < 8; ++j) load_to_lds16_if(true, ~0ull, src_a, off_a[j], dst + 16384 + j * 4096);
        advance(true);
    }
    wait_loads<24>(ns >= kRingStages);
    __syncthreads();
    RingFrags F0, F1;
    {
        const unsigned char *pa = ring + loff, *px = ring + 16384 + nh * 16384 + loff;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            F0.a[c] = *reinterpret_cast<const u32x4 *>(pa + c * 2048);
            F0.b[c] = *reinterpret_cast<const u32x4 *>(px + c * 2048);
        }
    }
    int buf = 0;                                                 // buffer of stage s
    auto step = [&](const RingFrags &cur, RingFrags &next, int s, bool new_group) __attribute__((always_inline)) {
        const int nbuf = buf == kRingStages - 1 ? 0 : buf + 1;
        wait_loads<12>(s + kRingStages <= ns);                   // stage s+2 may still be on its way
        __syncthreads();
        const bool go = s + kRingStages < ns;
        const uint32_t dst = wdst0 + buf * kRingStageBytes;
        // stage s+3 is the first half of a group in odd steps: its act rows
        if (new_group) rows_of_group(go ? (s + kRingStages) >> 1 : 0);
        __builtin_amdgcn_sched_barrier(0);
        {   // (in the last step this reads a stage that does not exist: in bounds, unused)
            const unsigned char *pa = ring + nbuf * kRingStageBytes + loff;
            const unsigned char *px = pa + 16384 + nh * 16384;
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                next.a[c] = *reinterpret_cast<const u32x4 *>(pa + c * 2048);
                next.b[c] = *reinterpret_cast<const u32x4 *>(px + c * 2048);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            load_to_lds16_if(go, ~0ull, src_a, off_a[c], dst + 16384 + c * 4096);
            if (c < 4) load_to_lds16_if(go, ~0ull, src_w, off_w[c], dst + c * 4096);
#pragma unroll
            for (int tt = 0; tt < 8; ++tt) mfma16_inplace(acc[c][tt], cur.a[c], cur.b[tt]);
            __builtin_amdgcn_sched_barrier(0);
        }
        advance(go);
        buf = nbuf;
    };
    for (int s = 0; s < ns; s += 2) {
        step(F0, F1, s, false);
        step(F1, F0, s + 1, true);
    }
    __syncthreads();                                             // every wave is done with the ring
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");           // the last matrix results are in the registers

    float *out = partial ? partial + (size_t)split * T * d : nullptr;
    if (ks == 0)
        down_finish<0>(acc, ring, wave, lane, t0 + nh * 128, T, d, j0, out, y);
    else
        down_finish<1>(acc, ring, wave, lane, t0 + nh * 128, T, d, j0, out, y);
}

// y = sum of the ranges' partial sums, added in the order of the ranges; n = T * d, a multiple of 8
__global__ __launch_bounds__(256) void reduce_partials(const float *__restrict__ partial, int splits, size_t n,
                                                       bf16_t *__restrict__ y)
{
    const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8;
    if (i >= n) return;
    float v[8];
    load8(partial + i, v);
    for (int k = 1; k < splits; ++k) {
        float w[8];
        load8(partial + (size_t)k * n + i, w);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] += w[e];
    }
    store8(y + i, v);
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
bool prefill_path_supported(int T, int d, int gs)
{
    // (the ring kernel addresses x rows with 32-bit byte offsets)
    return T > 1 && d % 128 == 0 && gs == 128 && (size_t)T * d * sizeof(bf16_t) < (1ull << 31);
}

hipError_t launch_ffn_prefill(const bf16_t *x, int T, int d, int G, int gs, const bf16_t *Wg,
                              const bf16_t *Wu, const bf16_t *Wd, const uint8_t *mask, bf16_t *y,
                              const DecodeScratch &ws, hipStream_t s)
{
    bf16_t *act = reinterpret_cast<bf16_t *>(ws.act);
    group_tokens_kernel<<<dim3(G), dim3(256), 0, s>>>(mask, T, G, ws.tok_list, ws.tok_cnt, ws.slot, act);
    static const hipError_t lds_ok = hipFuncSetAttribute(reinterpret_cast<const void *>(gate_up_pf_ring),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, kRingBytes);
    if (lds_ok != hipSuccess) return lds_ok;
    const int items_max = 2 * G * ((T + kRingTok - 1) / kRingTok);          // every group kept by every token
    launch_timed_lds("gate_up_pf_ring", gate_up_pf_ring, dim3((items_max + 7) / 8 * 8), dim3(256), kRingBytes, s, x, T,
                     d, G, Wg, Wu, (const int32_t *)ws.tok_list, (const int32_t *)ws.tok_cnt, act);
    const int splits = prefill_down_splits(T, d, G);
    if (splits == 0) {
        down_pf<<<dim3(d / 64, (T + 127) / 128), dim3(256), 0, s>>>(T, d, G, Wd, ws.slot, act, y);
        return hipGetLastError();
    }
    static const hipError_t lds_ok2 = hipFuncSetAttribute(reinterpret_cast<const void *>(down_pf_ring),
                                                          hipFuncAttributeMaxDynamicSharedMemorySize,
                                                          kRingBytes + kDownSlotBytes);
    if (lds_ok2 != hipSuccess) return lds_ok2;
    const int items = (d / 128) * ((T + kRingTok - 1) / kRingTok) * splits;
    float *partial = splits > 1 ? ws.partial : nullptr;
    down_pf_ring<<<dim3((items + 7) / 8 * 8), dim3(256), kRingBytes + kDownSlotBytes, s>>>(
        T, d, G, splits, Wd, (const int32_t *)ws.slot, (const int32_t *)ws.tok_cnt, (const bf16_t *)act, partial, y);
    if (splits > 1) {
        const size_t n = (size_t)T * d;
        reduce_partials<<<dim3((unsigned)((n / 8 + 255) / 256)), dim3(256), 0, s>>>(partial, splits, n, y);
    }
    return hipGetLastError();
}

}  // namespace halo
