// Deployment forward for T <= 16 tokens (Sec. 3.1 "Inference Latency": matrix-vector products bound
// by the weight bytes streamed from memory).  Y[t,i] = sum_g s[i,g] * sum_{k in g} X[t,k] (Q[i,k] - z[i,g]).
//
// Every packed word is read from HBM exactly once, straight into registers: a wave owns 128 output
// channels (lane (c, q): channel block c, feature block q of each 32-feature step) and walks a slice
// of the input features; the up-to-16 token rows ride along as the 16-row operand of MFMA 16x16x32,
// so T = 1 and T = 16 cost the same weight traffic.  Codes enter the MFMAs as exact bf16 (16 + Q);
// a ninth MFMA per step against a fragment of ones yields the row sums of X over the same features,
// and at the end of every scale group   y += s * (acc - (16 + z) * rowsum)   folds offset, zero-point
// and scale in fp32.  Per-channel layers are one group spanning the whole slice.
//
// Grid: one workgroup per (layer, channel tile of 128, feature slice); up to GEMV_MAX_LAYERS layers of different
// shapes and inputs share a launch (a decoder block's linears: a single LLaMA-size layer at such T is too short
// to fill the machine, and a launch costs as much as streaming several megabytes).  The K / 64 rounds of 64
// features of a tile are dealt evenly to its S slices and, inside a slice, to the waves of the workgroup (a wave
// may start or stop in the middle of a scale group: the fold above is linear in the features, so it is applied
// to whatever part of a group the wave has seen); the waves are summed through LDS at the end.
// S > 1 leaves fp32 partials [S, T, N] in the workspace for gemv_finish_kernel to add up in a fixed
// order.  Two shapes of workgroup: 4 waves (two or three workgroups per compute unit, S chosen so that
// the machine is full), and, for per-channel layers of 128 to 256 channel tiles, 12 waves that take
// the whole of K (S = 1): the same twelve waves per compute unit, but the sum over the feature ranges
// stays in LDS, so there are no partials and no second launch.  (With fewer tiles than that the
// compute units left idle cost more than the second launch saves: measured.)
//
// A wave moves its operands in rounds of 64 features (two MFMA steps): the packed blocks of its 16
// channel-block rows and the matching 128 bytes of each of the 16 token rows, by global -> LDS DMA
// into a private double buffer, from which each lane reads back its own blocks and activation
// fragments.  The LDS placement is chosen for conflict-free read-back: at 4 bits every lane's two
// 16-byte block halves sit at 16 * lane of two 1 KB planes per step; at 3 bits the 96 16-byte
// chunks of a step lie in address order (rows of 96 B).  No barrier is involved: a wave waits for
// its own DMA only.
#include <stddef.h>

#include <type_traits>

#include "peqa_device.h"
#include "peqa_kernels.h"

namespace peqa {

namespace {

constexpr int GV_WAVES = 4;          // waves of the sliced workgroup
constexpr int GV_WAVES_WHOLE = 12;   // waves of the workgroup that takes all of K
constexpr int GV_WHOLE_MIN_TILES = 128, GV_WHOLE_MAX_TILES = 256;
constexpr int GV_MAX_PER = 16;       // most scale groups a slice may touch (bounds the scale tile in LDS): trained zero-points
constexpr int NB_PC = 2, NB_G31 = 2; // ring depth of the per-channel instantiations / of the 3-bit group-wise one for T <= 8
constexpr int GV_MAX_PER_Z8 = 48;    // the same with integer zero-points, kept as bytes (5 instead of 8 bytes per entry)
// One round of one wave in LDS: its packed blocks (4 KB at 4 bits, 3 KB at 3 bits), then NX KB of token rows
// (8 rows x 128 B per KB: one DMA when T <= 8, two otherwise).
constexpr int gv_b_bytes(int bits) { return bits == 4 ? 4096 : 3072; }
constexpr int gv_round_bytes(int bits, int nx) { return gv_b_bytes(bits) + nx * 1024; }


__device__ __forceinline__ void gv_dma16(uint32_t voff, const void *sbase, uint32_t lds_dst)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(sbase), "s"(lds_dst) : "memory");
}
template <int N>
__device__ __forceinline__ void gv_wait_vmcnt()
{
    __builtin_amdgcn_s_waitcnt((N & 0xF) | (0x7 << 4) | (0xF << 8) | ((N >> 4) << 14));
}

// GROUPS_MAX: most scale groups a workgroup may touch: 1 for per-channel layers (1 KB scale tile),
// GV_MAX_PER for group-wise ones (16 KB).  NBUF: rounds a wave keeps in flight (its private ring in LDS).
// NX: KB of token rows per round (1: T <= 8, 2: T <= 16).
// ZBYTE: zero-points are the stored integers (no trained offset dz): they stay bytes in LDS, which lets a
// workgroup hold the scales of GV_MAX_PER_Z8 groups -- a whole row of LLaMA-13B's 40 -- and take all of K.
template <int BITS, int GROUPS_MAX, int WAVES, int NBUF, int NX, bool ZBYTE>
__global__ __launch_bounds__(WAVES * 64, WAVES > 4 ? 1 : 2) void gemv_kernel(GemvArgs a)
{
    // [wave][NBUF rounds][round]; reused as [wave][column tile][row][lane] fp32 (8 KB per wave) for the final sum
    extern __shared__ __align__(16) uint8_t stage[];
    // scale s0 + ds and zero-point (16 + z0 + dz as fp32, or z0 as stored) of [group of the slice][channel]
    // (rows padded: the transposing writes of consecutive groups of one channel then fall into different banks)
    __shared__ __align__(16) float sS[GROUPS_MAX][128 + 4];
    __shared__ __align__(16) typename std::conditional<ZBYTE, uint8_t, float>::type sZ[GROUPS_MAX][128 + (ZBYTE ? 8 : 4)];
    constexpr int WPB = 2 * BITS;
    constexpr int GV_B_BYTES = gv_b_bytes(BITS), GV_ROUND_BYTES = gv_round_bytes(BITS, NX);
    static_assert(NBUF * GV_ROUND_BYTES >= 8192, "the final sum reuses a wave's ring");
    constexpr int NDMA_B = 2 * 64 * WPB * 4 / 1024;               // 1 KB DMAs for the blocks of a round: 4 / 3
    constexpr int NDMA = NDMA_B + NX;                             // + the token rows
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, q = lane >> 4;
    // which layer this workgroup belongs to, and that layer's descriptor: scalar loads from the argument block
    const int bx = blockIdx.x;
    int li = 0, wg0 = 0;
#pragma unroll
    for (int i = 0; i < GEMV_MAX_LAYERS - 1; ++i) {
        const int e = kernarg_load<int>((uint32_t)(i * sizeof(GemvLayer) + offsetof(GemvLayer, wg_end)));
        if (bx >= e) { li = i + 1; wg0 = e; }
    }
    const GemvLayer L = kernarg_load<GemvLayer>((uint32_t)(li * sizeof(GemvLayer)));
    const uint32_t *l_packed = L.packed;
    const float *l_s0 = L.s0, *l_ds = L.ds, *l_dz = L.dz;
    const uint8_t *l_z0 = L.z0;
    uint16_t *l_Y = L.Y;
    const int l_N = L.N, l_S = L.S;
    const int tile = (int)((uint32_t)(bx - wg0) / (uint32_t)l_S), slice = (bx - wg0) - tile * l_S;
    const int n0 = tile * 128;                                   // first channel, within its layer
    const int K = L.K, G = L.G;
    const int chunk_rounds = L.chunk >> 6;                        // 64-feature rounds per scale group
    // this workgroup's rounds [rbeg, rend); wave w takes the w-th of WAVES equal parts of them
    const uint32_t R = (uint32_t)K >> 6;
    const int rbeg = (int)((uint32_t)slice * R / (uint32_t)l_S), rend = (int)((uint32_t)(slice + 1) * R / (uint32_t)l_S);
    const int wr0 = rbeg + (int)((uint32_t)(wave * (rend - rbeg)) / (uint32_t)WAVES);
    const int nrounds = rbeg + (int)((uint32_t)((wave + 1) * (rend - rbeg)) / (uint32_t)WAVES) - wr0;
    const int k0 = wr0 << 6;                                      // first feature of this wave
    const int g_lo = (uint32_t)rbeg / (uint32_t)chunk_rounds;     // first scale group this workgroup touches

    const uint32_t magic = kMagic;
    const u32x4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
    // the wave's tiles (128 channels x 32 features, TILE bytes each) are contiguous along the features
    constexpr uint32_t TILE = 64 * WPB * 4;
    const uint8_t *bbase = reinterpret_cast<const uint8_t *>(l_packed) +
                           ((size_t)tile * (K >> 5) + (k0 >> 5)) * TILE;
    const uint8_t *xbase = reinterpret_cast<const uint8_t *>(L.X + k0);
    const uint32_t lds_stage = (uint32_t)(uintptr_t)stage + wave * NBUF * GV_ROUND_BYTES;
    uint32_t b_voff[NDMA_B], x_voff[NX];
    if constexpr (BITS == 4) {
        // DMA (step s, half h): lane (c, q) fetches half h of its own block (c * 4 + q of tile s)
#pragma unroll
        for (int i = 0; i < NDMA_B; ++i)
            b_voff[i] = (uint32_t)(i >> 1) * TILE + (uint32_t)(c * 4 + q) * 32u + (uint32_t)(i & 1) * 16u;
    } else {
        // the 192 16-byte chunks of the round's two tiles, in address order
#pragma unroll
        for (int i = 0; i < NDMA_B; ++i) b_voff[i] = (uint32_t)(64 * i + lane) * 16u;
    }
#pragma unroll
    for (int i = 0; i < NX; ++i) {
        const int x = 64 * i + lane;                              // chunk x: token row x / 8, 16 bytes x % 8
        const int t = (x >> 3) < a.T ? (x >> 3) : a.T - 1;        // rows beyond T repeat the last one (never stored)
        x_voff[i] = (uint32_t)t * (uint32_t)K * 2u + (uint32_t)(x & 7) * 16u;
    }
    // round r lives in ring slot r % NBUF; `slot` is the slot of the next round to be issued
    int next_round = 0, slot = 0;
    auto issue_round = [&]() {
        const uint32_t dst = lds_stage + slot * GV_ROUND_BYTES;
        const uint8_t *bsrc = bbase + (size_t)next_round * 2 * TILE;   // two tiles per round
#pragma unroll
        for (int i = 0; i < NDMA_B; ++i) gv_dma16(b_voff[i], bsrc, dst + i * 1024);
        const uint8_t *xsrc = xbase + (size_t)next_round * 128;
#pragma unroll
        for (int i = 0; i < NX; ++i) gv_dma16(x_voff[i], xsrc, dst + GV_B_BYTES + i * 1024);
        ++next_round;
        slot = slot + 1 == NBUF ? 0 : slot + 1;
    };
#pragma unroll
    for (int i = 0; i < NBUF; ++i)
        if (i < nrounds) issue_round();

    // scale / zero-point tile of the slice: [groups touched][128 channels], transposed on the way into LDS (memory
    // has a channel's groups next to each other).  All loads of a thread are issued together (indices clamped
    // instead of branching, so that the compiler batches them behind a single wait); that wait also covers the
    // rounds above, which every wave needs next anyway.  idx / cols is taken in fp32 (exact: idx < 2^13).
    const int cols = (GROUPS_MAX > 1 && rend > rbeg) ? (int)((uint32_t)(rend - 1) / (uint32_t)chunk_rounds) - g_lo + 1 : 1;
    const float inv_cols = 1.0f / (float)cols;
    auto store_entry = [&](int jj, int ch, float sv, uint32_t zv, float dzv) {
        sS[jj][ch] = sv;
        if constexpr (ZBYTE) sZ[jj][ch] = (uint8_t)zv;
        else sZ[jj][ch] = kCodeOffset + (float)zv + dzv;
    };
    auto load_tile = [&](auto nb_c) {
        constexpr int NB = decltype(nb_c)::value;                 // batches of one entry per thread
        float ts[NB], td[NB], tdz[NB];
        uint8_t tz[NB];
        int ch[NB], jj[NB];
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int idx = tid + i * WAVES * 64;
            const bool on = idx < 128 * cols;
            ch[i] = on ? (int)(((float)idx + 0.5f) * inv_cols) : 0;
            jj[i] = on ? idx - ch[i] * cols : 0;
            const size_t si = (size_t)(n0 + ch[i]) * G + g_lo + jj[i];
            ts[i] = l_s0[si];
            tz[i] = l_z0[si];
            td[i] = l_ds ? l_ds[si] : 0.f;
            tdz[i] = l_dz ? l_dz[si] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < NB; ++i)
            if (tid + i * WAVES * 64 < 128 * cols) store_entry(jj[i], ch[i], ts[i] + td[i], tz[i], tdz[i]);
    };
    // A slice that spans all groups reads whole rows: the tile's entries are one contiguous run of 128 G, taken
    // four at a time (16 bytes of s0 and of ds, 4 bytes of z0 per thread and batch).
    auto load_rows = [&](auto nb_c) {
        constexpr int NB = decltype(nb_c)::value;                 // batches of four entries per thread
        f32x4 ts[NB], td[NB], tdz[NB];
        uint32_t tz[NB];
        const size_t base = (size_t)n0 * G;
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            int e = 4 * (tid + i * WAVES * 64);
            e = e < 128 * cols ? e : 0;
            ts[i] = *reinterpret_cast<const f32x4 *>(l_s0 + base + e);
            tz[i] = *reinterpret_cast<const uint32_t *>(l_z0 + base + e);
            td[i] = l_ds ? *reinterpret_cast<const f32x4 *>(l_ds + base + e) : f32x4{0.f, 0.f, 0.f, 0.f};
            tdz[i] = l_dz ? *reinterpret_cast<const f32x4 *>(l_dz + base + e) : f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int e = 4 * (tid + i * WAVES * 64);
            if (e < 128 * cols) {
                int chn = (int)(((float)e + 0.5f) * inv_cols), jn = e - chn * cols;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    store_entry(jn, chn, ts[i][u] + td[i][u], (tz[i] >> (8 * u)) & 0xFFu, tdz[i][u]);
                    if (++jn == cols) { jn = 0; ++chn; }
                }
            }
        }
    };
    constexpr int THREADS = WAVES * 64;
    if constexpr (GROUPS_MAX == 1) {
        load_tile(std::integral_constant<int, 1>{});
    } else if (cols == G) {
        // 128 cols / (4 THREADS) batches, at most GROUPS_MAX / 8 with 256 threads
        constexpr int NBMAX = (128 * GROUPS_MAX + 4 * THREADS - 1) / (4 * THREADS);
        if (128 * cols <= 4 * THREADS) load_rows(std::integral_constant<int, 1>{});
        else if (128 * cols <= 8 * THREADS || NBMAX <= 2) load_rows(std::integral_constant<int, NBMAX < 2 ? NBMAX : 2>{});
        else if (128 * cols <= 16 * THREADS || NBMAX <= 4) load_rows(std::integral_constant<int, NBMAX < 4 ? NBMAX : 4>{});
        else load_rows(std::integral_constant<int, NBMAX>{});
    } else {
        constexpr int PER_BATCH = THREADS / 128;                  // groups of 128 channels per batch of loads
        if (cols <= PER_BATCH) load_tile(std::integral_constant<int, 1>{});
        else if (cols <= 2 * PER_BATCH) load_tile(std::integral_constant<int, 2>{});
        else if (cols <= 4 * PER_BATCH) load_tile(std::integral_constant<int, 4>{});
        else if (cols <= 8 * PER_BATCH) load_tile(std::integral_constant<int, 8>{});
        else if constexpr (GROUPS_MAX > 8 * PER_BATCH) {
            if (cols <= 16 * PER_BATCH) load_tile(std::integral_constant<int, 16>{});
            else load_tile(std::integral_constant<int, (GROUPS_MAX + PER_BATCH - 1) / PER_BATCH>{});
        }
    }
    __syncthreads();

    f32x4 y[8], acc[8], accrs = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) { y[ct] = f32x4{0.f, 0.f, 0.f, 0.f}; acc[ct] = f32x4{0.f, 0.f, 0.f, 0.f}; }

    // this lane's block and activation fragment of step 0 within a round
    constexpr int STEP_B = BITS == 4 ? 2048 : 1536;               // packed bytes of one step in a round buffer
    const int b_off = BITS == 4 ? lane * 16 : c * 96 + q * 24;
    // token row of this lane's activation fragment; with 8 rows staged, rows 8..15 (beyond T, never stored) read rows 0..7
    const int x_off = GV_B_BYTES + (NX == 2 ? c : (c & 7)) * 128 + q * 16;
    int group_left = chunk_rounds - (int)((uint32_t)wr0 % (uint32_t)chunk_rounds);   // rounds to the end of the scale group
    int gj = (int)((uint32_t)wr0 / (uint32_t)chunk_rounds) - g_lo;                    // its column of the tile

    // One pass of this loop is one 32-feature MFMA step; it is deliberately a single copy of the
    // code (a workgroup runs only a few steps, so instruction fetch of an unrolled pipeline would
    // cost more than it hides).
    const int nsteps = 2 * nrounds;
    // Two workgroups share a compute unit, and its arbiter serves the older wave first: where the unit itself is
    // the limit, the workgroup dispatched first runs ahead, ends early, and leaves the other to finish alone with
    // half the loads in flight (measured: the first 256 workgroups of a launch ended 5 to 6 us before the rest).
    // The second one therefore takes the higher priority for the first half of its steps, the first one wins the
    // ties of the second half, and both end together.  Which workgroup came second is a guess from the index (the
    // first `second_from` are dealt one to every compute unit); a wrong guess costs time only.
    const bool second = bx >= a.second_from;
    if (second) __builtin_amdgcn_s_setprio(2);
    int rslot = 0;                                                // ring slot of the round being consumed
#pragma unroll 1
    for (int step = 0; step < nsteps; ++step) {
        const int r = step >> 1, s2 = step & 1;
        if (second && step == (nsteps >> 1)) __builtin_amdgcn_s_setprio(0);
        if (s2 == 0) {
            // rounds r .. min(r + NBUF, nrounds) - 1 are in flight, issued in order: wait for r only
            const int after = next_round - 1 - r;                 // rounds issued after r
            if (NBUF > 3 && after >= 3) gv_wait_vmcnt<3 * NDMA>();
            else if (NBUF > 2 && after == 2) gv_wait_vmcnt<2 * NDMA>();
            else if (after == 1) gv_wait_vmcnt<NDMA>();
            else gv_wait_vmcnt<0>();
            asm volatile("" ::: "memory");
        }
        const uint8_t *rb = stage + (wave * NBUF + rslot) * GV_ROUND_BYTES;
        {
            const uint8_t *sb = rb + s2 * STEP_B + b_off;
            uint32_t bw[WPB];
            if constexpr (BITS == 4) {
                const u32x4 v0 = *reinterpret_cast<const u32x4 *>(sb);
                const u32x4 v1 = *reinterpret_cast<const u32x4 *>(sb + 1024);
#pragma unroll
                for (int i = 0; i < 4; ++i) { bw[i] = v0[i]; bw[4 + i] = v1[i]; }
            } else {
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    const u32x2 v = *reinterpret_cast<const u32x2 *>(sb + 8 * i);
                    bw[2 * i] = v[0];
                    bw[2 * i + 1] = v[1];
                }
            }
            const u32x4 af = *reinterpret_cast<const u32x4 *>(rb + x_off + s2 * 64);
            BlockUnpacker<BITS, false> up;
            up.prepare(bw);
            u32x4 bf[8];
            bf[0] = up.template frag<0>(magic); bf[1] = up.template frag<1>(magic);
            bf[2] = up.template frag<2>(magic); bf[3] = up.template frag<3>(magic);
            bf[4] = up.template frag<4>(magic); bf[5] = up.template frag<5>(magic);
            bf[6] = up.template frag<6>(magic); bf[7] = up.template frag<7>(magic);
#pragma unroll
            for (int ct = 0; ct < 8; ++ct) acc[ct] = mfma16(af, bf[ct], acc[ct]);
            accrs = mfma16(af, ones, accrs);
        }
        if (s2 == 1) {
            // this buffer is free again (its LDS reads have returned: the MFMAs consumed them): refill it
            if (next_round < nrounds) issue_round();
            rslot = rslot + 1 == NBUF ? 0 : rslot + 1;
            if (--group_left == 0 || r + 1 == nrounds) {
                // end of a scale group, or of this wave's share: fold offset, zero-point and scale
                // of the group into y, restart the sums
                const f32x4 s_lo = *reinterpret_cast<const f32x4 *>(&sS[gj][8 * c]);
                const f32x4 s_hi = *reinterpret_cast<const f32x4 *>(&sS[gj][8 * c + 4]);
                float zo[8];                                      // 16 + z of channels 8c .. 8c + 7
                if constexpr (ZBYTE) {
                    const u32x2 zz = *reinterpret_cast<const u32x2 *>(&sZ[gj][8 * c]);
#pragma unroll
                    for (int i = 0; i < 8; ++i) zo[i] = kCodeOffset + (float)((zz[i >> 2] >> (8 * (i & 3))) & 0xFFu);
                } else {
                    const f32x4 z_lo = *reinterpret_cast<const f32x4 *>(&sZ[gj][8 * c]);
                    const f32x4 z_hi = *reinterpret_cast<const f32x4 *>(&sZ[gj][8 * c + 4]);
#pragma unroll
                    for (int i = 0; i < 4; ++i) { zo[i] = z_lo[i]; zo[4 + i] = z_hi[i]; }
                }
#pragma unroll
                for (int ct = 0; ct < 8; ++ct) {
                    const float sc = ct < 4 ? s_lo[ct & 3] : s_hi[ct & 3];
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) y[ct][jj] += sc * (acc[ct][jj] - zo[ct] * accrs[jj]);
                    acc[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
                accrs = f32x4{0.f, 0.f, 0.f, 0.f};
                ++gj;
                group_left = chunk_rounds;
            }
        }
    }

    // ---- sum the waves, then write Y (S = 1) or this slice's partial
    __syncthreads();                                              // everyone is done with the stage buffers
    float *red = reinterpret_cast<float *>(stage);                // [wave][column tile][row in lane][lane], 32 KB
#pragma unroll
    for (int ct = 0; ct < 8; ++ct)
#pragma unroll
        for (int j = 0; j < 4; ++j) red[((wave * 8 + ct) * 4 + j) * 64 + lane] = y[ct][j];
    __syncthreads();
    // the 8 column tiles x 4 rows x 64 lanes of results are dealt to the threads; each adds the waves in order
    for (int idx = tid; idx < 8 * 4 * 64; idx += WAVES * 64) {
        const int ct = idx >> 8, j = (idx >> 6) & 3, ln = idx & 63;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) v += red[((w * 8 + ct) * 4 + j) * 64 + ln];
        const int t = 4 * (ln >> 4) + j, n = n0 + 8 * (ln & 15) + ct;
        if (t < a.T) {
            if (l_S == 1) l_Y[(size_t)t * l_N + n] = (uint16_t)float_to_bf16_bits(v);
            else L.partial[((size_t)slice * a.T + t) * l_N + n] = v;
        }
    }
}

// Y[t,n] = bf16( partial[0][t,n] + partial[1][t,n] + ... ), fixed order, for every sliced layer of the launch
// (blockIdx.y = layer; layers with a single slice wrote their Y themselves).
__global__ __launch_bounds__(256) void gemv_finish_kernel(GemvArgs a)
{
    const GemvLayer L = kernarg_load<GemvLayer>((uint32_t)(blockIdx.y * sizeof(GemvLayer)));
    if (L.S == 1) return;
    // T <= 16 and at most 2^24 channels: everything fits 32-bit arithmetic
    const uint32_t tn = (uint32_t)a.T * (uint32_t)L.N;
    const uint32_t e = blockIdx.x * 256u + threadIdx.x;
    if (e >= tn) return;
    float v = 0.f;
    for (int sl = 0; sl < L.S; ++sl) v += L.partial[(size_t)sl * tn + e];
    L.Y[e] = (uint16_t)float_to_bf16_bits(v);
}

}  // namespace

int gemv_slices(int Ntot, int K, int T, int chunk, bool zbyte)
{
    // as many slices as give two workgroups per compute unit (measured: more, up to the three that fit
    // for per-channel layers, only adds partials), every wave at least two rounds long, and the
    // partials small next to the weight bytes
    const int tiles = Ntot / 128, R = K / 64, chunk_rounds = chunk / 64;
    // per-channel layers that fill half to all of the compute units with one tile each: one 12-wave
    // workgroup per tile takes all of K
    if (chunk == K && tiles >= GV_WHOLE_MIN_TILES && tiles <= GV_WHOLE_MAX_TILES) return 1;
    int S = 512 / tiles;
    // between one and one and a half tiles per compute unit a single slice leaves the units with one
    // 4-wave workgroup each: two slices (up to three workgroups per unit) stream better, partials included
    if (chunk == K && tiles > GV_WHOLE_MAX_TILES && 2 * tiles <= 768) S = 2;
    if (S > R / (2 * GV_WAVES)) S = R / (2 * GV_WAVES);
    const int by_bytes = T > 4 ? 6 : 16;
    if (S > by_bytes) S = by_bytes;
    if (S < 1) S = 1;
    // the scale tile in LDS holds a bounded number of groups per slice
    const int gmax = zbyte ? GV_MAX_PER_Z8 : GV_MAX_PER;
    if (chunk != K)
        while (((R + S - 1) / S + chunk_rounds - 1) / chunk_rounds + 1 > gmax) ++S;
    return S;
}

bool gemv_whole(int tiles, bool per_channel, int S)
{
    return per_channel && S == 1 && tiles >= GV_WHOLE_MIN_TILES && tiles <= GV_WHOLE_MAX_TILES;
}

void gemv_plan(int n, const int *N, const int *K, const int *chunk, int bits, int T, bool zbyte, int *S)
{
    // target: all workgroups resident at once (two per compute unit) with equal shares of the packed bytes.
    // Per-channel layers at T <= 4: three per compute unit (they fit, with 1 KB of scales each).  A channel tile
    // of a 4096-feature layer is two thirds of a compute unit's share of a LLaMA-7B block, so whole tiles load
    // the units 2 : 1; halves deal out evenly, and at such T their partial sums are a few per cent of the bytes
    // (measured on that block: 7 % less time at T = 1, 2 % more at T = 16).
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    double total = 0.0;
    bool per_channel_all = true;
    for (int j = 0; j < n; ++j) {
        total += (double)N[j] * K[j] * bits / 8.0;
        per_channel_all = per_channel_all && chunk[j] == K[j];
    }
    const double target = total / ((per_channel_all && T <= 4 ? 3.0 : 2.0) * cus);
    const int by_bytes = T > 4 ? 6 : 16;                         // partials stay small next to the weight bytes
    for (int j = 0; j < n; ++j) {
        const int R = K[j] / 64, chunk_rounds = chunk[j] / 64;
        const double tile_bytes = 128.0 * K[j] * bits / 8.0;
        int s = (int)(tile_bytes / target + 0.5);
        if (s > R / (2 * GV_WAVES)) s = R / (2 * GV_WAVES);      // every wave at least two rounds
        if (s > by_bytes) s = by_bytes;
        if (s < 1) s = 1;
        // the scale tile in LDS holds a bounded number of groups per slice
        const int gmax = zbyte ? GV_MAX_PER_Z8 : GV_MAX_PER;
        if (chunk[j] != K[j])
            while (((R + s - 1) / s + chunk_rounds - 1) / chunk_rounds + 1 > gmax) ++s;
        S[j] = s;
    }
}

hipError_t launch_gemv(int bits, const GemvArgs &a_in, hipStream_t stream)
{
    const int wgs = a_in.layer[a_in.n_layers - 1].wg_end;
    GemvArgs a = a_in;
    {
        int d = 0, cus = 256;
        if (hipGetDevice(&d) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, d);
        a.second_from = cus;
    }
    bool per_channel_all = true, sliced = false;
    unsigned max_tn = 0;
    for (int j = 0; j < a.n_layers; ++j) {
        per_channel_all = per_channel_all && a.layer[j].chunk == a.layer[j].K;
        sliced = sliced || a.layer[j].S > 1;
        if (a.layer[j].S > 1 && (unsigned)a.T * (unsigned)a.layer[j].N > max_tn) max_tn = (unsigned)a.T * (unsigned)a.layer[j].N;
    }
    const dim3 grid(wgs);
    // the 12-wave form: layers of equal K in one launch (one layer, or layers that read one X), a single slice each
    bool whole = !sliced && gemv_whole(wgs, per_channel_all, 1);
    for (int j = 1; j < a.n_layers; ++j) whole = whole && a.layer[j].K == a.layer[0].K;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    // One instantiation: its dynamic LDS (more than the default limit: allowed once per device), then the launch.
    auto go = [&](auto kern, int waves, int lds_bytes, bool *allowed) -> hipError_t {
        if (!allowed[dev]) {
            const hipError_t e2 = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                      hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
            if (e2 != hipSuccess) return e2;
            allowed[dev] = true;
        }
        trace_before(KID_GEMV, stream);
        hipLaunchKernelGGL(kern, grid, dim3(waves * 64), lds_bytes, stream, a);
        trace_after(KID_GEMV, stream);
        return hipGetLastError();
    };
#define PEQA_GEMV_GO(BITS, GROUPS, WAVES, NBUF, NX, ZBYTE)                                                \
    do {                                                                                                   \
        static bool allowed[64];                                                                           \
        e = go(gemv_kernel<BITS, GROUPS, WAVES, NBUF, NX, ZBYTE>, WAVES, WAVES * NBUF * gv_round_bytes(BITS, NX), allowed); \
    } while (0)
    const bool nx2 = a.T > 8;
    bool zbyte = true;
    for (int j = 0; j < a.n_layers; ++j) zbyte = zbyte && a.layer[j].dz == nullptr;
    if (whole) {
        if (bits == 4) PEQA_GEMV_GO(4, 1, GV_WAVES_WHOLE, 2, 2, false); else PEQA_GEMV_GO(3, 1, GV_WAVES_WHOLE, 2, 2, false);
    } else if (per_channel_all) {
        if (bits == 4) { if (nx2) PEQA_GEMV_GO(4, 1, GV_WAVES, NB_PC, 2, false); else PEQA_GEMV_GO(4, 1, GV_WAVES, NB_PC, 1, false); }
        else { if (nx2) PEQA_GEMV_GO(3, 1, GV_WAVES, NB_PC, 2, false); else PEQA_GEMV_GO(3, 1, GV_WAVES, NB_PC, 1, false); }
    } else if (zbyte) {
        if (bits == 4) { if (nx2) PEQA_GEMV_GO(4, GV_MAX_PER_Z8, GV_WAVES, 2, 2, true); else PEQA_GEMV_GO(4, GV_MAX_PER_Z8, GV_WAVES, 2, 1, true); }
        else { if (nx2) PEQA_GEMV_GO(3, GV_MAX_PER_Z8, GV_WAVES, 2, 2, true); else PEQA_GEMV_GO(3, GV_MAX_PER_Z8, GV_WAVES, NB_G31, 1, true); }
    } else {
        if (bits == 4) { if (nx2) PEQA_GEMV_GO(4, GV_MAX_PER, GV_WAVES, 2, 2, false); else PEQA_GEMV_GO(4, GV_MAX_PER, GV_WAVES, 2, 1, false); }
        else { if (nx2) PEQA_GEMV_GO(3, GV_MAX_PER, GV_WAVES, 2, 2, false); else PEQA_GEMV_GO(3, GV_MAX_PER, GV_WAVES, 2, 1, false); }
    }
#undef PEQA_GEMV_GO
    if (e != hipSuccess || !sliced) return e;
    trace_before(KID_GEMV_FINISH, stream);
    hipLaunchKernelGGL(gemv_finish_kernel, dim3((max_tn + 255) / 256, a.n_layers), dim3(256), 0, stream, a);
    trace_after(KID_GEMV_FINISH, stream);
    return hipGetLastError();
}

}  // namespace peqa
