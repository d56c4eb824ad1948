// Dense contractions of the PEQA linear layer on gfx950 MFMA (per-channel scales).
//
//   MODE_Y   : Y[t,i]    = s_i * sum_k X[t,k] (Q[i,k] - z_i)                (Eq. 2 forward)
//   MODE_DDS : part[i]   = sum_{t in tile} dY[t,i] * sum_k X[t,k] (Q[i,k] - z_i)
//                                                   (scale gradient, column-reduced epilogue)
//   MODE_DX  : dX[t,k]   = sum_i (dY[t,i] s_i) (Q[i,k] - z_i)                (chain rule on Eq. 2)
//
// One workgroup = 8 waves = a 128 (tokens) x 256 (output columns) tile.  Waves are laid out
// 2 (token halves) x 2 (column halves) x 2 (halves of the contraction range): every wave owns a
// 64 x 128 accumulator (4 x 8 MFMA 16x16x32 tiles, 128 fp32 AGPRs) over its half of the
// contraction.  Two waves share each SIMD, so that the LDS reads, the unpacking and the scalar
// bookkeeping of one hide behind the matrix instructions of the other; the contraction split
// keeps 256 workgroups busy on a 2048 x 4096 output.  The two halves are summed through LDS in
// the epilogue (or, for MODE_DDS, after the column reduction, which is linear).
// A second form (KW = 1) runs four waves (2 x 2) over the whole contraction range of the same tile with half
// the ring, two workgroups per compute unit: launches with more than one tile per compute unit take it (see
// halves_per_workgroup below).  Its loop is unrolled by the ring depth.  The scale gradient and dX of one
// per-channel backward run as four-wave tiles of one launch (gemm_bwd_pair_kernel); in the group-wise dX
// launch, spare workgroups at the end of the grid write the transposed operands of the token contraction.
//
// Operand paths.  Both operands go global -> LDS by DMA (global_load_lds) into a ring of
// stages, one 32-deep contraction step per stage: the activation operand (X, or the pre-scaled
// dY) as two 128 x 32 bf16 tiles (16-byte chunks XOR-swizzled by row), the weight operand as
// the packed 8x8 code blocks themselves, one per lane.  Each lane reads its block back and
// unpacks it in registers into bf16 (16 + Q) fragments (peqa_device.h): dequantised weights
// never exist in memory.  The contraction therefore runs on exact small integers; the offset 16,
// the zero-point and the scale are applied in the epilogue from row sums of the other
// operand:   sum_k X (Q - z) = sum_k X (16 + Q) - (16 + z) sum_k X.
//
// Group-wise scales (Sec. 4.2 and Table 5; group size a multiple of 64) use the GROUPED instantiations:
//   MODE_Y, MODE_DX : the scale cannot leave the contraction, so every weight enters the MFMA as
//                     bf16( s[i,g] (Q[i,k] - z[i,g]) ), formed in fp32 from a per-group table of
//                     (s, -s (16 + z)) that rides through LDS next to the operand ring; the
//                     epilogue is a plain store and the activation operand is X / dY itself.
//   MODE_DDS        : one workgroup contracts one pair of scale groups (blockIdx.y), each
//                     contraction half one group, and the column-reduced epilogue writes one
//                     partial per (token tile, channel, group).  This is the older of two routes to
//                     the grouped scale gradient (the default contracts over tokens, peqa_dw.hip)
//                     and runs only on request (option grouped_dds = 1).
#include <stddef.h>

#include <type_traits>

#include "peqa_device.h"
#include "peqa_kernels.h"

namespace peqa {

namespace {

constexpr int TILE_T = 128;
constexpr int TILE_C = 256;
constexpr int KSTEP = 32;                                  // contraction depth of one loop iteration
constexpr int NSTAGE = 6;                                  // LDS ring depth
constexpr int A_HALF_BYTES = TILE_T * KSTEP * 2;           // 8 KB: 128 rows x 32 bf16 of one contraction half
constexpr int B_WAVE_BYTES = 2048;                         // one packed 8x8 block per lane (32 B / 24 B)
// A ring stage holds, per contraction half the workgroup runs (KW = 2 or 1), one 128 x 32 activation tile and
// the packed weights of the two column halves: 24 KB or 12 KB.
constexpr int stage_bytes(int kw) { return kw * (A_HALF_BYTES + 2 * B_WAVE_BYTES); }
constexpr int DMA_PER_ITER = 3;                            // DMA instructions per wave per iteration
constexpr int ring_bytes(int kw) { return NSTAGE * stage_bytes(kw); }   // 144 KB (the epilogue's exchange of 128 KB reuses it) or 72 KB
constexpr int tbl_bytes(int kw) { return 2 * kw * 2 * 1024; }           // grouped MODE_Y / MODE_DX: 2 x 1 KB of (s, b) per (column half, contraction half);
                                                                        // twice that for MODE_DX when groups end inside a 128-feature run

// One tile of one contraction: the work of workgroup number `wg` of a launch of this contraction alone.
// ASCALE (group-wise dX in the four-wave form, group size a multiple of 128, integer zero-points): every wave's 128
// feature columns lie in one scale group g, so the scale s[i, g] varies along the contraction only and is applied to the
// activation fragments in registers, A_g[t,i] = bf16(dY[t,i] s[i,g]): 16 registers per step instead of the 32 of the
// weight fragments.  The codes are contracted as the exact integers 16 + Q, as in the per-channel kernels, and the
// zero-point term crow[t] = sum_i A_g[t,i] (16 + z[i,g]) is added up beside the matrix instructions from the same
// rounded fragments (one dot2 per register against the exact bf16 of 16 + z), so that it cancels the code offset.
template <int BITS, int MODE, bool GROUPED, int KW, bool ASCALE = false>
__device__ __forceinline__ void gemm_tile(const GemmArgs &a, const int wg, uint8_t *lds)
{
    constexpr int STAGE_BYTES = stage_bytes(KW);
    constexpr int WPB = 2 * BITS;                          // words per 8x8 block
    constexpr bool ALONG_CH = (MODE == MODE_DX);           // contraction over output channels
    constexpr bool SCALED = GROUPED && MODE != MODE_DDS;   // the scale is applied inside the loop
    constexpr bool WSCALED = SCALED && !ASCALE;            // ... to the weights: they enter the MFMA already scaled
    constexpr bool PAIRED = GROUPED && MODE == MODE_DDS;   // one scale group per contraction half
    static_assert(!ASCALE || (GROUPED && MODE == MODE_DX && KW == 1), "activation-side scaling is a form of the four-wave group-wise dX");
    static_assert(KW == 2 || (KW == 1 && !PAIRED), "the paired scale gradient needs both contraction halves");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in an SGPR
    const int wt = wave & 1, wn = (wave >> 1) & 1, wk = KW == 2 ? wave >> 2 : 0;   // token half, column half, contraction half
    const int c = lane & 15, q = lane >> 4;

    // workgroup -> tile.  Workgroup ids are dealt round-robin to the 8 XCDs and every CU holds one
    // workgroup, so the 32 ids {x, x + 8, ...} that run together on XCD x are given one patch of
    // patch_t x (32 / patch_t) neighbouring tiles: they share activation rows and weight columns
    // through that XCD's L2 instead of each pulling its own from the fabric.
    int tile_t, tile_c;
    {
        const int xcd = wg & 7, local = wg >> 3;
        const int g = (local >> 5) * 8 + xcd;              // patch number
        const int r = local & 31;                          // position in the patch
        const int pt = a.patch_t, patches_t = (a.tiles_t + pt - 1) / pt;
        tile_t = (g % patches_t) * pt + (r % pt);
        tile_c = (g / patches_t) * (32 / pt) + (r / pt);
    }
    if (tile_t >= a.tiles_t || tile_c >= a.tiles_c) return;   // padding of a ragged patch (uniform per workgroup)

    const int t0 = tile_t * TILE_T;
    const int col0 = tile_c * TILE_C + wn * 128;           // first output column of this wave
    const bool wave_on = col0 < a.C;
    const int T = a.T, KC = a.KC;
    // contraction ranges of the two halves: [kh0, kh0 + 32 nit) and [kh1, kh1 + 32 nit)
    int kh0, kh1, nit, grp = 0;
    bool half_on = true;
    if constexpr (PAIRED) {
        // groups 2 y and 2 y + 1; with an odd number of groups the last workgroup's second half
        // re-reads its first group and drops the result
        const int g1 = 2 * (int)blockIdx.y + 1;
        kh0 = 2 * (int)blockIdx.y * a.gsz;
        kh1 = (g1 < a.G ? g1 : g1 - 1) * a.gsz;
        nit = a.gsz / KSTEP;                               // >= 2 and even: the group size is a multiple of 64
        grp = 2 * (int)blockIdx.y + wk;
        half_on = grp < a.G;
    } else if constexpr (KW == 2) {
        kh0 = 0;
        kh1 = KC >> 1;                                     // both waves of a column half take KC/2
        nit = kh1 / KSTEP;                                 // loop iterations (>= 2: KC % 128 == 0)
    } else {
        kh0 = kh1 = 0;
        nit = KC / KSTEP;                                  // a multiple of 4
    }
    const int kbeg = wk ? kh1 : kh0;
    const uint32_t magic = kMagic;
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;

    // ---- activation tiles: global -> LDS by DMA, 16 wave-loads of 1 KB per iteration (2 per wave).
    // Wave-load m = 8 i + wave covers contraction half m / 8, rows 16 (m % 8) .. +16; lane s lands at
    // byte 16 s of that 1 KB, i.e. row s / 4, chunk position s % 4, and fetches the chunk that the
    // XOR swizzle assigns to that position.
    // With a single contraction half the four waves fetch the tile's 128 rows in two wave-loads each:
    // rows 16 wave .. and 64 + 16 wave .. (the swizzle only looks at row % 16).
    uint32_t a_voff, a_voff_hi = 0;
    {
        const int row_l = lane >> 2, pos = lane & 3;
        const int chunk = pos ^ a_swizzle(row_l);
        auto voff_of = [&](int row) __attribute__((always_inline)) {
            row = t0 + row < T ? row : T - 1 - t0;
            return (uint32_t)row * (uint32_t)KC * 2u + (uint32_t)chunk * 16u;
        };
        a_voff = voff_of(wave * 16 + row_l);
        if constexpr (KW == 1) a_voff_hi = voff_of(64 + wave * 16 + row_l);
    }
    const uint8_t *a_base = reinterpret_cast<const uint8_t *>(a.A) + (size_t)t0 * KC * 2;

    // ---- packed weights: one 8x8 block per lane per iteration, also by DMA, into the slot shared by
    // the two token-half waves of this (column half, contraction half); each of them fetches half of it
    // along features: lane (c, q) owns channel block col0/8 + c and feature block 4 it + q
    // along channels: lane (c, q) owns feature block col0/8 + c and channel block 4 it + q
    // Blocks are stored in tiles of 16 channel blocks x 4 feature blocks (TILE bytes), tiles along the
    // features first.  Along features a step of a wave is exactly one tile; along channels it is a
    // quarter (4 channel blocks x 4 feature blocks, contiguous) of each of 4 neighbouring tiles.
    constexpr uint32_t BLK = WPB * 4, TILE = 64 * BLK;
    const size_t tile_row = (size_t)(a.K >> 5) * TILE;     // bytes per row of tiles
    const uint8_t *b_base;
    const int m0 = kbeg >> 5;                              // 32-deep contraction step at which this wave starts
    uint32_t b_voff, b_voff2 = 0;
    int b_lane_off;                                        // where this lane's block sits in the wave's LDS slot
    if constexpr (!ALONG_CH)
        b_base = reinterpret_cast<const uint8_t *>(a.packed) + (size_t)(col0 >> 7) * tile_row + (size_t)m0 * TILE;
    else
        b_base = reinterpret_cast<const uint8_t *>(a.packed) + (size_t)(col0 >> 5) * TILE;
    if constexpr (BITS == 4) {
        // two DMAs of 16 B per lane: the halves of the lane's own 32-byte block
        b_voff = ALONG_CH ? (uint32_t)(c >> 2) * TILE + (uint32_t)(q * 4 + (c & 3)) * BLK : (uint32_t)(c * 4 + q) * BLK;
        b_lane_off = lane * 16;
    } else {
        // 24-byte blocks: the wave's 64 blocks are 1536 contiguous bytes (along features) or 4 runs of
        // 384 B, one per tile (along channels) = 96 chunks of 16 B, fetched as chunk `lane` and chunk
        // `64 + lane` and laid down in LDS in chunk order.
        const int x0 = lane, x1 = 64 + (lane & 31);
        if constexpr (!ALONG_CH) {
            b_voff = (uint32_t)x0 * 16u;
            b_voff2 = (uint32_t)x1 * 16u;
            b_lane_off = (c * 4 + q) * 24;
        } else {
            b_voff = (uint32_t)(x0 / 24) * TILE + (uint32_t)(x0 % 24) * 16u;
            b_voff2 = (uint32_t)(x1 / 24) * TILE + (uint32_t)(x1 % 24) * 16u;
            b_lane_off = (c >> 2) * 384 + (q * 4 + (c & 3)) * 24;
        }
    }
    if (!wave_on) { b_voff = lane * 32; b_voff2 = lane * 32; }
    // Packed bytes of this wave's contraction steps.  They are fetched strictly in order, one step per call
    // (the last one again and again once the range is used up; a wave without columns re-reads tile 0), so a
    // running pointer advanced with selects stands in for the address arithmetic: branches in the loop cost
    // the wave's instruction stream more than the few scalar operations.
    const uint8_t *b_next = reinterpret_cast<const uint8_t *>(a.packed);
    if (wave_on) b_next = ALONG_CH ? b_base + (size_t)(m0 >> 2) * tile_row + (size_t)(m0 & 3) * (16 * BLK) : b_base;
    int b_idx = 0;                                         // step b_next points at
    auto b_advance = [&]() __attribute__((always_inline)) {
        const bool more = wave_on && b_idx < nit - 1;
        size_t inc = TILE;
        if constexpr (ALONG_CH) inc = ((m0 + b_idx) & 3) == 3 ? tile_row - 3 * (size_t)(16 * BLK) : (size_t)(16 * BLK);
        b_next += more ? inc : 0;
        b_idx += more ? 1 : 0;
    };
    const int slot = wn + 2 * wk;
    if constexpr (BITS == 3) { if (wt) b_voff = b_voff2; }

    // One of the three DMAs of a step: 0, 1 = activation tile (contraction half 0, 1; or, with one half, rows
    // 0..63 and 64..127), 2 = packed weights.
    // 4-bit weights: the two 16-byte halves of every lane's block go to the two token-half waves;
    // 3-bit: chunks 0..63 and 64..95 of the slot (lanes 32..63 of the second repeat chunks 64..95
    // into the slot's unused tail).
    auto issue_one = [&](int which, int it, int stage) __attribute__((always_inline)) {
        const uint32_t sb = lds_base + stage * STAGE_BYTES;
        if (which < 2) {
            if constexpr (KW == 2)
                dma16(a_voff, a_base + (size_t)it * KSTEP * 2 + (size_t)(which ? kh1 : kh0) * 2,
                      sb + which * A_HALF_BYTES + wave * 1024);
            else
                dma16(which ? a_voff_hi : a_voff, a_base + (size_t)it * KSTEP * 2, sb + which * (A_HALF_BYTES / 2) + wave * 1024);
        } else {
            const uint8_t *bp = b_next + (BITS == 4 ? wt * 16 : 0);   // `it` is implied: the calls come in step order
            dma16(b_voff, bp, sb + KW * A_HALF_BYTES + slot * B_WAVE_BYTES + wt * 1024);
            b_advance();
        }
    };
    auto issue = [&](int it, int stage) __attribute__((always_inline)) {
        issue_one(0, it, stage);
        issue_one(1, it, stage);
        issue_one(2, it, stage);
    };

    // ---- grouped MODE_Y / MODE_DX: (s, b = -s (16 + z)) of 128 channels of one scale group, 1 KB,
    // fetched by DMA one block of steps ahead into a double buffer behind the ring, by the first
    // token-half wave of every (column half, contraction half).  Steps m are counted from the start
    // of the layer's contraction range.
    //   along features: block B = steps m with m >> bshift == B, i.e. 128 features -- or 64 when the
    //                   group size is not a multiple of 128 (`fine`); the wave's 128 channels, group
    //                   of those features
    //   along channels: block B = steps 4 B .. 4 B + 3 = channels 128 B .. 128 B + 127, group of the
    //                   wave's feature columns; when `fine`, columns 0..63 and 64..127 of the wave may
    //                   lie in two groups: two chunks per block, the second fetched by the second
    //                   token-half wave, and lanes pick theirs by column half
    const bool fine = SCALED && (a.gsz & 127) != 0;
    const int bshift = (!ALONG_CH && fine) ? 1 : 2;
    const uint32_t tbuf = (ALONG_CH && fine) ? 2048 : 1024;    // bytes per buffer
    const uint32_t tbl_off = NSTAGE * STAGE_BYTES + slot * 2 * tbuf;
    auto issue_table = [&](int B) __attribute__((always_inline)) {
        const int last = (KC >> (5 + bshift)) - 1;
        B = B < last ? B : last;
        const size_t g = ALONG_CH ? (size_t)((col0 + (fine ? 64 * wt : 0)) / a.gsz) : (size_t)((B << (5 + bshift)) / a.gsz);
        const size_t ch = ALONG_CH ? (size_t)B << 7 : (size_t)col0;
        // (s, b) pairs of 128 channels, 1 KB; with activation-side scaling the 1 KB of block B: its 128 scales, then its
        // 128 offsets 16 + z as bf16 (exact), then padding
        const uint8_t *src = reinterpret_cast<const uint8_t *>(a.sb) +
                             (wave_on ? (ASCALE ? (g * (size_t)(a.N >> 7) + (size_t)B) * 1024 : (g * a.N + ch) * 8) : 0);
        dma16(lane * 16, src, lds_base + tbl_off + (B & 1) * tbuf + ((ALONG_CH && fine) ? wt * 1024 : 0));
    };
    const bool table_wave = wt == 0 || (ALONG_CH && fine);
    // The next block is fetched at the step m with (m & tbl_mask) == tbl_phase: its second step when a block has four,
    // its first when it has two; never by the other waves.  Both wave-uniform, and said so, which makes the test one
    // scalar compare that keeps no vector register.
    // (Along channels the same form costs registers instead: the plain test stays there.)
    const int tbl_mask = (1 << bshift) - 1;
    const int tbl_phase = ALONG_CH ? 0 : __builtin_amdgcn_readfirstlane(table_wave ? (bshift == 2 ? 1 : 0) : -1);
    auto next_table_at = [&](int m) __attribute__((always_inline)) -> bool {
        if constexpr (ALONG_CH) return (m & tbl_mask) == (bshift == 2 ? 1 : 0) && table_wave;
        else return (m & tbl_mask) == tbl_phase;
    };
    // Entries of contraction step m for this lane's 8 block channels: along features 8 c .. 8 c + 7 of
    // block m / 4, along channels 32 (m % 4) + 8 q .. + 7.  Along channels every fragment needs all
    // eight (element e of a fragment is channel e): they are read into registers once per step.
    // Along features fragment I needs only entry I: it is read when the fragment's first register is
    // built, which keeps 14 registers free.
    float sc[8], bo[8];
    uint32_t zf[4];                                        // ASCALE: 16 + z of the same channels as exact bf16 pairs
    float crow_acc[4] = {0.f, 0.f, 0.f, 0.f};              // ASCALE: this lane's part of crow of token rows 16 rt + c
    const uint8_t *tbl_row = nullptr;
    auto read_table = [&](int m) __attribute__((always_inline)) {
        if constexpr (ASCALE) {
            // scales and offsets of channels 32 (m % 4) + 8 q .. + 7 of the block.  (The step after the last one reads the
            // last one's: a buffer that has been written, whatever the number of blocks.)
            m = m < m0 + nit ? m : m0 + nit - 1;
            tbl_row = lds + tbl_off + ((m >> 2) & 1) * tbuf + (m & 3) * 128 + q * 32;
            const f32x4 lo = *reinterpret_cast<const f32x4 *>(tbl_row), hi = *reinterpret_cast<const f32x4 *>(tbl_row + 16);
            const u32x4 zv = *reinterpret_cast<const u32x4 *>(lds + tbl_off + ((m >> 2) & 1) * tbuf + 512 + (m & 3) * 64 + q * 16);
#pragma unroll
            for (int e = 0; e < 4; ++e) { sc[e] = lo[e]; sc[4 + e] = hi[e]; zf[e] = zv[e]; }
            return;
        }
        tbl_row = lds + tbl_off + ((m >> bshift) & 1) * tbuf +
                  (ALONG_CH ? (fine ? (c >> 3) * 1024 : 0) + (m & 3) * 256 + q * 64 : c * 64);
        if constexpr (ALONG_CH) {
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                const f32x4 v = *reinterpret_cast<const f32x4 *>(tbl_row + 16 * h);
                sc[2 * h] = v[0]; bo[2 * h] = v[1]; sc[2 * h + 1] = v[2]; bo[2 * h + 1] = v[3];
            }
        }
    };
    // register J of fragment I of the next step: plain (16 + Q) pairs, or scaled weights
    auto next_frag_reg = [&](const BlockUnpacker<BITS, ALONG_CH> &up, auto i_c, auto j_c) __attribute__((always_inline)) -> uint32_t {
        constexpr int I = decltype(i_c)::value, J = decltype(j_c)::value;
        const uint32_t pr = up.template frag_reg<I, J>(magic);
        if constexpr (!WSCALED) {
            return pr;
        } else if constexpr (!ALONG_CH) {
            if constexpr (J == 0) {
                const f32x2 v = *reinterpret_cast<const f32x2 *>(tbl_row + 8 * I);
                sc[0] = v[0];
                bo[0] = v[1];
            }
            return scale_pair(pr, sc[0], bo[0], sc[0], bo[0]);
        } else {
            return scale_pair(pr, sc[2 * J], bo[2 * J], sc[2 * J + 1], bo[2 * J + 1]);
        }
    };

    // ASCALE: the activation fragment of row tile rt (8 contraction elements 8 q .. 8 q + 7 of a step) times the
    // step's scales, and its part of the zero-point term
    auto scale_a = [&](u32x4 &f, int rt) __attribute__((always_inline)) {
#pragma unroll
        for (int J = 0; J < 4; ++J) {
            f[J] = mul_pair(f[J], sc[2 * J], sc[2 * J + 1]);
            crow_acc[rt] = dot2_bf16(f[J], zf[J], crow_acc[rt]);
        }
    };

    f32x4 acc[4][8];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // row = 64 wt + 16 rt + c and the swizzle only looks at row % 16
    const int a_read_off = wk * A_HALF_BYTES + (64 * wt + c) * 64 + ((q ^ a_swizzle(c)) << 4);
    const int b_read_off = KW * A_HALF_BYTES + slot * B_WAVE_BYTES + b_lane_off;
    auto read_b = [&](int stage, uint32_t *bw) __attribute__((always_inline)) {
        const uint8_t *st = lds + stage * STAGE_BYTES + b_read_off;
        if constexpr (BITS == 4) {
            const u32x4 v0 = *reinterpret_cast<const u32x4 *>(st);
            const u32x4 v1 = *reinterpret_cast<const u32x4 *>(st + 1024);
#pragma unroll
            for (int i = 0; i < 4; ++i) { bw[i] = v0[i]; bw[4 + i] = v1[i]; }
        } else {
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                const u32x2 v = *reinterpret_cast<const u32x2 *>(st + 8 * i);
                bw[2 * i] = v[0];
                bw[2 * i + 1] = v[1];
            }
        }
    };

    auto read_a = [&](int stage, u32x4 *afrag, int rt) __attribute__((always_inline)) {
        afrag[rt] = *reinterpret_cast<const u32x4 *>(lds + stage * STAGE_BYTES + a_read_off + rt * 16 * 64);
    };

    // ---- prologue: queue NSTAGE - 1 stages, wait for the first three, fetch the operands of step 0
    // and the packed weights of step 1
    u32x4 bfrag[2][8], afrag[4];
    uint32_t bw[2][WPB];                                   // packed weights of the next step / the one after
    if constexpr (SCALED) {
        if (table_wave) { issue_table(m0 >> bshift); issue_table((m0 >> bshift) + 1); }
    }
#pragma unroll
    for (int sidx = 0; sidx < NSTAGE - 1; ++sidx) issue(sidx < nit ? sidx : nit - 1, sidx);
    issue_one(2, NSTAGE - 1 < nit ? NSTAGE - 1 : nit - 1, NSTAGE - 1);   // the packed weights run one stage further ahead
    wait_vmcnt<DMA_PER_ITER *(NSTAGE - 4) + 1>();
    __syncthreads();
    {
        read_b(0, bw[1]);
        read_b(1, bw[0]);
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) read_a(0, afrag, rt);
        if constexpr (SCALED) read_table(m0);
        if constexpr (ASCALE) {
#pragma unroll
            for (int rt = 0; rt < 3; ++rt) scale_a(afrag[rt], rt);   // the fourth: in step 0 (see scale_next)
        }
        BlockUnpacker<BITS, ALONG_CH> up;
        up.prepare(bw[1]);
        static_for<8>([&](auto i) {
            static_for<4>([&](auto j) { bfrag[0][i.value][j.value] = next_frag_reg(up, i, j); });
        });
    }
    // step 0 refills the packed-weight slot of stage 0, which the partner wave may still be reading
    __syncthreads();

    // ---- main loop.  A step is a 32-deep contraction: 32 MFMAs, one per accumulator.  When step
    // `it` starts, its fragments and the packed weights of step it + 1 are in registers, and stages
    // it + 1 and it + 2 are complete in LDS.  The MFMAs run back to back from the first instruction
    // after the barrier; everything else sits in their shadow, in fixed slots:
    //   after every MFMA      one register of step it + 1's weight fragments (shift + and_or)
    //   after MFMA 2          LDS read of the packed weights of step it + 2
    //   after MFMA 5, 13, 21  one DMA each: the two activation tiles of step it + NSTAGE - 1 (into the
    //                         stage of step it - 1) and the packed weights of step it + NSTAGE (into
    //                         this step's own stage: they were read two steps ago, and they are the
    //                         operand that comes from HBM, so they get the longer lead).  The tail
    //                         re-fetches the last tile: harmless, and it keeps the DMA count per step
    //                         constant so that a fixed vmcnt tells when a stage has landed
    //   after each 8 MFMAs    the activation fragment just used up is refilled from LDS for step it + 1
    // NSTAGE steps per loop trip, so that the ring stage of every step is a compile-time constant: LDS
    // destinations and read offsets are then literals.  With the stage in a register, forty-odd scalar
    // instructions of ring and address arithmetic ran at the top of every step, which every wave went through
    // right after the barrier and before its first matrix instruction (in a test loop of the same instruction
    // mix forty dependent scalar instructions at that place cost 0.11 us per step; in this kernel taking them
    // out gained 1-2 %).  What is left per step is one running source pointer for the activation tiles, one for
    // the packed weights, and the step counter.
    static_assert(NSTAGE % 2 == 0, "the register buffers alternate with the step's parity");
    // LDS reads take a 16-bit literal offset: the stages of the first and of the second half of the ring are
    // addressed from one lane-dependent base register each (kept live across the loop), the rest is literal.
    constexpr int HALF_RING = (NSTAGE / 2) * STAGE_BYTES;
    static_assert((NSTAGE / 2 - 1) * STAGE_BYTES + 4096 <= 65536, "literal offsets of LDS reads");
    const uint8_t *a_rd[2] = {lds + a_read_off, lds + a_read_off + HALF_RING};
    const uint8_t *b_rd[2] = {lds + b_read_off, lds + b_read_off + HALF_RING};
    auto read_a_st = [&](auto st_c, u32x4 *af, int rt) __attribute__((always_inline)) {
        constexpr int ST = decltype(st_c)::value;
        af[rt] = *reinterpret_cast<const u32x4 *>(a_rd[ST / (NSTAGE / 2)] + (ST % (NSTAGE / 2)) * STAGE_BYTES + rt * 16 * 64);
    };
    auto read_b_st = [&](auto st_c, uint32_t *w) __attribute__((always_inline)) {
        constexpr int ST = decltype(st_c)::value;
        const uint8_t *st = b_rd[ST / (NSTAGE / 2)] + (ST % (NSTAGE / 2)) * STAGE_BYTES;
        if constexpr (BITS == 4) {
            const u32x4 v0 = *reinterpret_cast<const u32x4 *>(st);
            const u32x4 v1 = *reinterpret_cast<const u32x4 *>(st + 1024);
#pragma unroll
            for (int i = 0; i < 4; ++i) { w[i] = v0[i]; w[4 + i] = v1[i]; }
        } else {
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                const u32x2 v = *reinterpret_cast<const u32x2 *>(st + 8 * i);
                w[2 * i] = v[0];
                w[2 * i + 1] = v[1];
            }
        }
    };
    const uint8_t *a_ptr = a_base + (size_t)(NSTAGE - 1 < nit ? NSTAGE - 1 : nit - 1) * KSTEP * 2 + (KW == 2 ? (size_t)kh0 * 2 : 0);
    const uint32_t a_voff_2 = KW == 2 ? a_voff + (uint32_t)(kh1 - kh0) * 2u : a_voff_hi;   // second activation DMA, same source pointer
    const uint32_t dst_a = lds_base + wave * 1024;
    const uint32_t dst_b = lds_base + KW * A_HALF_BYTES + slot * B_WAVE_BYTES + wt * 1024;
    // ASCALE: a fragment is scaled one row tile after its read was issued, when its data has arrived (scaling the one
    // just read would stall the wave for the LDS latency four times a step): after the matrix instructions of row
    // tile rt >= 1 of step `it`, the fragment of row tile rt - 1 of step it + 1.  Row tile 3's fragment, read at the end
    // of the step before, is scaled at the top of its own step, before that step fetches the scales of the next.
    // The last step does the same with the fragments it reads for the step after it (a tile of real data, re-fetched
    // by the tail of the ring: finite values), which are never contracted: what they added to crow is taken out
    // again after the loop (take_out_phantom), which keeps branches and a second copy of the step out of the loop.
    constexpr bool RING_UNROLL_C = !SCALED || (WSCALED && KW == 1 && !(ALONG_CH && BITS == 4));   // see below
    auto scale_next = [&](auto rt_c) __attribute__((always_inline)) {
        constexpr int rt = decltype(rt_c)::value;
        if constexpr (rt >= 1) scale_a(afrag[rt - 1], rt - 1);
    };
    auto take_out_phantom = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int rt = 0; rt < 3; ++rt) {
            float p = 0.f;
#pragma unroll
            for (int J = 0; J < 4; ++J) p = dot2_bf16(afrag[rt][J], zf[J], p);
            crow_acc[rt] -= p;
        }
    };
    // (inlined by force: ten copies are more than the inliner takes by itself, and a call would pass the
    // captured scalars through memory)
    auto step = [&](int it, auto stage_c) __attribute__((always_inline)) {
        constexpr int S = decltype(stage_c)::value;             // LDS stage of this step
        constexpr int CUR = S & 1, NXT = CUR ^ 1;
        constexpr int NS = (S + 1) % NSTAGE;                    // stage of step it + 1
        constexpr int NNS = (S + 2) % NSTAGE;                   // stage of step it + 2
        constexpr int PS = (S + NSTAGE - 1) % NSTAGE;           // stage of step it - 1 = of step it + NSTAGE - 1
        if constexpr (ASCALE) {
            scale_a(afrag[3], 3);
            __builtin_amdgcn_sched_barrier(0);             // the old scales die before the new ones are read
        }
        if constexpr (SCALED) {
            // the fragments built in this step belong to contraction step m = m0 + it + 1
            const int m = m0 + it + 1;
            read_table(m);
            // The buffer of the block before m's was last read in the previous step: fetch the block
            // after m's into it.  With blocks of four steps this is done at the block's second step
            // (three steps of lead); with blocks of two, at its first (two steps: the DMA is complete
            // after the next step's wait and visible after its barrier, just in time).
            if (next_table_at(m)) issue_table((m >> bshift) + 1);
        }
        BlockUnpacker<BITS, ALONG_CH> up;
        up.prepare(bw[CUR]);
        static_for<4>([&](auto rt_c) {
            constexpr int rt = rt_c.value;
            static_for<8>([&](auto ct_c) {
                constexpr int ct = ct_c.value, m = 8 * rt + ct;
                mfma16_acc(acc[rt][ct], afrag[rt], bfrag[CUR][ct]);
                bfrag[NXT][2 * rt + (ct >> 2)][ct & 3] =
                    next_frag_reg(up, std::integral_constant<int, 2 * rt + (ct >> 2)>{}, std::integral_constant<int, (ct & 3)>{});
                if constexpr (m == 2) read_b_st(std::integral_constant<int, NNS>{}, bw[NXT]);
                if constexpr (m == 5) dma16(a_voff, a_ptr, dst_a + PS * STAGE_BYTES);
                if constexpr (m == 13) dma16(a_voff_2, a_ptr, dst_a + PS * STAGE_BYTES + (KW == 2 ? A_HALF_BYTES : A_HALF_BYTES / 2));
                if constexpr (m == 21) {
                    dma16(b_voff, b_next + (BITS == 4 ? wt * 16 : 0), dst_b + S * STAGE_BYTES);
                    b_advance();
                    // the activation tiles of the next step's DMAs: one step further, until the range is used up
                    a_ptr += it + NSTAGE - 1 < nit - 1 ? KSTEP * 2 : 0;
                }
            });
            read_a_st(std::integral_constant<int, NS>{}, afrag, rt);
            static_assert(!ASCALE || !RING_UNROLL_C, "activation-side scaling runs the two-step loop");
        });
        // Own DMA for step it + 3 has landed; the barrier makes every wave's part visible.
        // No wait on LDS reads is needed here: what this step read is overwritten two steps later.
        wait_vmcnt<DMA_PER_ITER *(NSTAGE - 4) + 1>();
        bare_barrier();
    };
    // The grouped forward / dX (scaled fragments) in its eight-wave form, and one instantiation of its four-wave
    // form, do not fit into their registers when unrolled that far -- the compiler spills inside the loop, which
    // the hand-counted DMA queue cannot take -- and keep the stage in a register, two steps per trip (the
    // register buffers alternate).  For the eight-wave per-channel kernels the unrolled loop measures the same
    // as the other (within 0.3 %): their loss against the four-wave form is ring fill, exchange and epilogue,
    // which nothing overlaps with one workgroup per compute unit.
    constexpr bool RING_UNROLL = RING_UNROLL_C;
    if constexpr (RING_UNROLL) {
        int it = 0;
        for (; it + NSTAGE <= nit; it += NSTAGE)
            static_for<NSTAGE>([&](auto s_c) { step(it + decltype(s_c)::value, s_c); });
        // nit is even (KC % 128 == 0): none, two or four steps are left, in stages 0..3
        if (nit - it >= 2) {
            step(it, std::integral_constant<int, 0>{});
            step(it + 1, std::integral_constant<int, 1>{});
        }
        if (nit - it >= 4) {
            step(it + 2, std::integral_constant<int, 2>{});
            step(it + 3, std::integral_constant<int, 3>{});
        }
    } else {
    int cur = 0;                                           // LDS stage of the current step
    auto step2 = [&](int it, auto cur_c) __attribute__((always_inline)) {
        constexpr int CUR = decltype(cur_c)::value, NXT = CUR ^ 1;
        const int pre = it + NSTAGE - 1 < nit ? it + NSTAGE - 1 : nit - 1;
        const int pre_b = it + NSTAGE < nit ? it + NSTAGE : nit - 1;
        const int nstage = cur + 1 == NSTAGE ? 0 : cur + 1;       // stage of step it + 1
        const int nnstage = nstage + 1 == NSTAGE ? 0 : nstage + 1; // stage of step it + 2
        const int pstage = cur == 0 ? NSTAGE - 1 : cur - 1;       // stage of step it - 1 = of step it + NSTAGE - 1
        if constexpr (ASCALE) {
            scale_a(afrag[3], 3);
            __builtin_amdgcn_sched_barrier(0);             // the old scales die before the new ones are read
        }
        if constexpr (SCALED) {
            // the fragments built in this step belong to contraction step m = m0 + it + 1
            const int m = m0 + it + 1;
            read_table(m);
            // The buffer of the block before m's was last read in the previous step: fetch the block
            // after m's into it.  With blocks of four steps this is done at the block's second step
            // (three steps of lead); with blocks of two, at its first (two steps: the DMA is complete
            // after the next step's wait and visible after its barrier, just in time).
            if (next_table_at(m)) issue_table((m >> bshift) + 1);
        }
        BlockUnpacker<BITS, ALONG_CH> up;
        up.prepare(bw[CUR]);
        static_for<4>([&](auto rt_c) {
            constexpr int rt = rt_c.value;
            static_for<8>([&](auto ct_c) {
                constexpr int ct = ct_c.value, m = 8 * rt + ct;
                mfma16_acc(acc[rt][ct], afrag[rt], bfrag[CUR][ct]);
                bfrag[NXT][2 * rt + (ct >> 2)][ct & 3] =
                    next_frag_reg(up, std::integral_constant<int, 2 * rt + (ct >> 2)>{}, std::integral_constant<int, (ct & 3)>{});
                if constexpr (m == 2) read_b(nnstage, bw[NXT]);
                if constexpr (m == 5) issue_one(0, pre, pstage);
                if constexpr (m == 13) issue_one(1, pre, pstage);
                if constexpr (m == 21) issue_one(2, pre_b, cur);
            });
            read_a(nstage, afrag, rt);
            if constexpr (ASCALE) scale_next(rt_c);
        });
        // Own DMA for step it + 3 has landed; the barrier makes every wave's part visible.
        // No wait on LDS reads is needed here: what this step read is overwritten two steps later.
        wait_vmcnt<DMA_PER_ITER *(NSTAGE - 4) + 1>();
        bare_barrier();
        cur = nstage;
    };
    for (int it = 0; it < nit; it += 2) {                  // nit is even: KC % 128 == 0
        step2(it, std::integral_constant<int, 0>{});
        step2(it + 1, std::integral_constant<int, 1>{});
    }
    }
    if constexpr (ASCALE) take_out_phantom();
    // The loop's exits meet here; this keeps the accumulators in their AGPRs past that point (the compiler would
    // otherwise copy all 128 of them into VGPRs at once, more than there are)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) asm volatile("" : "+a"(acc[i][j]));
    // ASCALE: the lanes (c, 0..3) hold the four feature-block parts of crow of token row 16 rt + c: add them (fixed
    // order); every lane of the four then has the row's total
    if constexpr (ASCALE) {
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) {
            crow_acc[rt] += __shfl_xor(crow_acc[rt], 16);
            crow_acc[rt] += __shfl_xor(crow_acc[rt], 32);
        }
    }
    // The epilogue works out its lane indices afresh (from a copy of the thread index that the compiler cannot
    // connect to the first one), so that none of them has to be held in a register through the loop.
    {
    int tid_e = threadIdx.x;
    asm volatile("" : "+v"(tid_e));
    const int tid = tid_e, lane = tid & 63, c = lane & 15, q = lane >> 4;
    // Epilogue parameters are fetched while the last DMAs drain: per-column scale and zero-point of
    // this lane's 8 columns, per-row correction terms of the 8 rows this wave finishes (MODE_Y, MODE_DX)
    // correction term of row 4 q + j of this wave's row tile rt: the row sum of X (MODE_Y) or crow (MODE_DX)
    auto row_term = [&](int rt, int j) __attribute__((always_inline)) -> float {
        int t = t0 + 64 * wt + rt * 16 + 4 * q + j;
        t = t < T ? t : T - 1;
        if constexpr (MODE == MODE_Y) {
            const u32x2 r2 = *reinterpret_cast<const u32x2 *>(a.rs + 2 * t);
            return __uint_as_float(r2[0]) + __uint_as_float(r2[1]);
        } else if constexpr (MODE == MODE_DX) {
            if constexpr (ASCALE) return __shfl(crow_acc[rt], 4 * q + j);   // row 16 rt + 4 q + j: from lane c = 4 q + j
            else return a.crow[t];
        } else {
            return 0.f;
        }
    };
    float ep_sc[8], ep_zoff[8], ep_row[8];
    if (wave_on && !WSCALED) {
        if constexpr (PAIRED) {
            const int g = half_on ? grp : a.G - 1;
#pragma unroll
            for (int ct = 0; ct < 8; ++ct) ep_zoff[ct] = kCodeOffset + (float)a.z0[(size_t)(col0 + 8 * c + ct) * a.G + g];
            if (a.dz) {
#pragma unroll
                for (int ct = 0; ct < 8; ++ct) ep_zoff[ct] += a.dz[(size_t)(col0 + 8 * c + ct) * a.G + g];
            }
        } else if constexpr (MODE != MODE_DX) {
            const u32x2 zz = *reinterpret_cast<const u32x2 *>(a.z0 + col0 + 8 * c);
#pragma unroll
            for (int ct = 0; ct < 8; ++ct) ep_zoff[ct] = kCodeOffset + (float)((zz[ct >> 2] >> (8 * (ct & 3))) & 0xFFu);
            if (a.dz) {
                const f32x4 z_lo = *reinterpret_cast<const f32x4 *>(a.dz + col0 + 8 * c);
                const f32x4 z_hi = *reinterpret_cast<const f32x4 *>(a.dz + col0 + 8 * c + 4);
#pragma unroll
                for (int ct = 0; ct < 4; ++ct) { ep_zoff[ct] += z_lo[ct]; ep_zoff[4 + ct] += z_hi[ct]; }
            }
        }
        if constexpr (MODE == MODE_Y) {
            const f32x4 s_lo = *reinterpret_cast<const f32x4 *>(a.s0 + col0 + 8 * c);
            const f32x4 s_hi = *reinterpret_cast<const f32x4 *>(a.s0 + col0 + 8 * c + 4);
#pragma unroll
            for (int ct = 0; ct < 4; ++ct) { ep_sc[ct] = s_lo[ct]; ep_sc[4 + ct] = s_hi[ct]; }
            if (a.ds) {
                const f32x4 d_lo = *reinterpret_cast<const f32x4 *>(a.ds + col0 + 8 * c);
                const f32x4 d_hi = *reinterpret_cast<const f32x4 *>(a.ds + col0 + 8 * c + 4);
#pragma unroll
                for (int ct = 0; ct < 4; ++ct) { ep_sc[ct] += d_lo[ct]; ep_sc[4 + ct] += d_hi[ct]; }
            }
        }
        if constexpr (MODE != MODE_DDS) {
#pragma unroll
            for (int i = 0; i < 8; ++i) ep_row[i] = row_term(2 * wk + (i >> 2), i & 3);
        }
    }
    wait_vmcnt<0>();
    __syncthreads();
    mfma_result_fence();

    // ---- epilogues
    if constexpr (MODE == MODE_DDS) {
        // column sums of dY[t,i] * (acc[t,i] - (16 + z_i) * rowsum_half[t]) over the tile's rows
        float colsum[8];
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) colsum[ct] = 0.f;
        if (wave_on) {
            // This lane's 16 rows are t0 + 64 wt + 16 rt + 4 q + j.  Rows past T are clamped for the
            // loads and masked in the sum, so that all loads are unconditional: dY and the row sums
            // four rows at a time, the next four in flight while these are used.
            auto row_of = [&](int rt, int j) __attribute__((always_inline)) { return t0 + 64 * wt + rt * 16 + 4 * q + j; };
            u32x4 dyv[2][4];
            float rsv[2][4];
            auto load_rows = [&](auto rt_c, u32x4 *dst, float *rdst) __attribute__((always_inline)) {
                constexpr int rt = decltype(rt_c)::value;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int t = row_of(rt, j), tc = t < T ? t : T - 1;
                    dst[j] = *reinterpret_cast<const u32x4 *>(a.dY + (size_t)tc * a.C + col0 + 8 * c);
                    // row sum of X over this contraction half, or over this half's scale group
                    if constexpr (PAIRED) {
                        rdst[j] = a.rs[(size_t)tc * a.G + (half_on ? grp : a.G - 1)];
                    } else if constexpr (KW == 2) {
                        rdst[j] = a.rs[2 * tc + wk];
                    } else {
                        const u32x2 r2 = *reinterpret_cast<const u32x2 *>(a.rs + 2 * tc);
                        rdst[j] = __uint_as_float(r2[0]) + __uint_as_float(r2[1]);
                    }
                }
            };
            load_rows(std::integral_constant<int, 0>{}, dyv[0], rsv[0]);
            static_for<4>([&](auto rt_c) {
                constexpr int rt = rt_c.value;
                if constexpr (rt + 1 < 4) load_rows(std::integral_constant<int, rt + 1>{}, dyv[(rt + 1) & 1], rsv[(rt + 1) & 1]);
                float dm[4];                                   // rows past T contribute nothing
#pragma unroll
                for (int j = 0; j < 4; ++j) dm[j] = row_of(rt, j) < T ? 1.f : 0.f;
#pragma unroll
                for (int ct = 0; ct < 8; ++ct) {
                    // one accumulator tile at a time leaves its AGPRs
                    const f32x4 av = read_acc(acc[rt][ct]);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint32_t w = dyv[rt & 1][j][ct >> 1];
                        const float d = ((ct & 1) ? bf16_hi(w) : bf16_lo(w)) * dm[j];
                        colsum[ct] += d * (av[j] - ep_zoff[ct] * rsv[rt & 1][j]);
                    }
                }
            });
        }
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) {
            colsum[ct] += __shfl_xor(colsum[ct], 16);
            colsum[ct] += __shfl_xor(colsum[ct], 32);
        }
        float *red = reinterpret_cast<float *>(lds);           // [waves][128]
        if (q == 0) {
#pragma unroll
            for (int ct = 0; ct < 8; ++ct) red[wave * 128 + 8 * c + ct] = colsum[ct];
        }
        __syncthreads();
        if (tid < 256) {
            const int w2 = tid >> 7, col = tid & 127;          // column half, column in half
            const int n = tile_c * TILE_C + tid;
            // waves wt + 2 wn + 4 wk of this column half, in a fixed order
            const float *r0 = red + (2 * w2) * 128 + col;
            if constexpr (PAIRED) {
                // the two contraction halves are two scale groups: one partial each
                const int g0 = 2 * (int)blockIdx.y;
                if (n < a.C) {
                    float *dst = a.partial + ((size_t)tile_t * a.C + n) * a.G + g0;
                    dst[0] = r0[0] + r0[128];
                    if (g0 + 1 < a.G) dst[1] = r0[4 * 128] + r0[5 * 128];
                }
            } else if constexpr (KW == 2) {
                if (n < a.C)
                    a.partial[(size_t)tile_t * a.C + n] = (r0[0] + r0[128]) + (r0[4 * 128] + r0[5 * 128]);
            } else {
                if (n < a.C) a.partial[(size_t)tile_t * a.C + n] = r0[0] + r0[128];
            }
        }
    } else {
        // rows 4 q + j (j = 0..3) of row tile rt, whose sums over the whole contraction are in sum[ct][j];
        // r[j] = their correction terms
        auto store_rows = [&](int rt, const f32x4 *sum, const float *r_) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int t = t0 + 64 * wt + rt * 16 + 4 * q + j;
                if (t < T) {
                    float v[8];
                    const float r = r_[j];
                    if constexpr (WSCALED) {
#pragma unroll
                        for (int ct = 0; ct < 8; ++ct) v[ct] = sum[ct][j];
                    } else if constexpr (MODE == MODE_Y) {
#pragma unroll
                        for (int ct = 0; ct < 8; ++ct) v[ct] = sum[ct][j] - ep_zoff[ct] * r;
                        if (a.P) {                         // keep the unscaled product for the backward
                            f32x4 *dst = reinterpret_cast<f32x4 *>(a.P + (size_t)t * a.C + col0 + 8 * c);
                            dst[0] = f32x4{v[0], v[1], v[2], v[3]};
                            dst[1] = f32x4{v[4], v[5], v[6], v[7]};
                        }
#pragma unroll
                        for (int ct = 0; ct < 8; ++ct) v[ct] *= ep_sc[ct];
                    } else {
#pragma unroll
                        for (int ct = 0; ct < 8; ++ct) v[ct] = sum[ct][j] - r;
                    }
                    u32x4 o;
#pragma unroll
                    for (int p = 0; p < 4; ++p) o[p] = pack_bf16x2(v[2 * p], v[2 * p + 1]);
                    *reinterpret_cast<u32x4 *>(a.out + (size_t)t * a.C + col0 + 8 * c) = o;
                }
            }
        };
        if constexpr (KW == 1) {
            // one contraction range per workgroup: every wave holds the finished sums of its four row tiles;
            // the correction terms of the last two are fetched while the first two are stored
            if (wave_on) {
                float ep_row_hi[8];
                if constexpr (!WSCALED) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) ep_row_hi[i] = row_term(2 + (i >> 2), i & 3);
                }
#pragma unroll
                for (int rt = 0; rt < 4; ++rt) {
                    f32x4 sum[8];
#pragma unroll
                    for (int ct = 0; ct < 8; ++ct) sum[ct] = acc[rt][ct];
                    store_rows(rt, sum, rt < 2 ? ep_row + 4 * rt : ep_row_hi + 4 * (rt - 2));
                }
            }
        } else {
        // sum the two contraction halves: wave wk keeps row tiles [2 wk, 2 wk + 2) and sends the others
        f32x4 *xch = reinterpret_cast<f32x4 *>(lds);           // [8 waves][16 tiles][64 lanes]
        auto finish = [&](auto keep_c) __attribute__((always_inline)) {
            constexpr int KEEP = decltype(keep_c)::value;      // first row tile this wave keeps
            constexpr int SEND = 2 - KEEP;
            {
                f32x4 *mine = xch + (size_t)wave * 16 * 64 + lane;
#pragma unroll
                for (int rtl = 0; rtl < 2; ++rtl)
#pragma unroll
                    for (int ct = 0; ct < 8; ++ct) mine[(rtl * 8 + ct) * 64] = acc[SEND + rtl][ct];
            }
            __syncthreads();
            if (!wave_on) return;
            const f32x4 *theirs = xch + (size_t)(wave ^ 4) * 16 * 64 + lane;
#pragma unroll
            for (int rtl = 0; rtl < 2; ++rtl) {
                f32x4 sum[8];
#pragma unroll
                for (int ct = 0; ct < 8; ++ct) sum[ct] = read_acc(acc[KEEP + rtl][ct]) + theirs[(rtl * 8 + ct) * 64];
                store_rows(KEEP + rtl, sum, ep_row + 4 * rtl);
            }
        };
        if (wk == 0) finish(std::integral_constant<int, 0>{});
        else finish(std::integral_constant<int, 2>{});
        }
    }
    }
}

template <int BITS, int MODE, bool GROUPED, int KW, bool ASCALE = false>
__global__ __launch_bounds__(256 * KW, 3 - KW) void gemm_kernel(GemmArgs a)
{
    extern __shared__ __align__(16) uint8_t lds[];
    if constexpr (MODE == MODE_DX && GROUPED && KW == 1) {
        // Workgroups past the tiles: an independent, bandwidth-bound job of the same backward -- the transposed
        // copies of X and dY that the token contraction (the scale gradient, launched next) reads.  They are
        // dispatched last and take the places that the last tiles leave free on the compute units, so most of
        // their time is not added to the launch.
        const int spare = (int)blockIdx.x - ((int)gridDim.x - a.tp_blocks);
        if (spare >= 0) {
            const int bts = a.tp_Tp >> 6, nx = bts * (a.K >> 6);
            uint16_t(*tile)[64 + 2] = reinterpret_cast<uint16_t(*)[64 + 2]>(lds);
            if (spare < nx) transpose_pad_tile(a.tp_X, a.T, a.K, a.tp_Xt, spare % bts, spare / bts, tile);
            else transpose_pad_tile(a.A, a.T, a.N, a.tp_dYt, (spare - nx) % bts, (spare - nx) / bts, tile);
            return;
        }
    }
    gemm_tile<BITS, MODE, GROUPED, KW, ASCALE>(a, (int)blockIdx.x, lds);
}

// Both contractions of a per-channel backward in one launch of four-wave workgroups: the first n_first
// workgroups are the tiles of one of them (the one with the longer contraction), the rest the tiles of the
// other.  Neither reads what the other writes.  Two launches of at most one tile per compute unit each -- which
// would run in the eight-wave form, ring fill and epilogue exposed, or leave most of the machine idle at small T --
// become one launch with up to two workgroups per compute unit, and the last round of the first contraction is
// filled with tiles of the second.
template <int BITS>
__global__ __launch_bounds__(256, 2) void gemm_bwd_pair_kernel(GemmArgs a_dds, GemmArgs a_dx, int n_first, int dx_first)
{
    extern __shared__ __align__(16) uint8_t lds[];
    const int b = (int)blockIdx.x;
    const bool first = b < n_first;
    const int wg = first ? b : b - n_first;
    if (first == (dx_first != 0)) gemm_tile<BITS, MODE_DX, false, 1>(a_dx, wg, lds);
    else gemm_tile<BITS, MODE_DDS, false, 1>(a_dds, wg, lds);
}

// Bandwidth-bound side work inside a multi-contraction launch: auxiliary workgroup `w` of `m.aux_wgs` walks the
// units w, w + aux_wgs, ... of one index space: first the SDY_ROWS-row blocks of the scale_dy jobs, then the
// 256-element chunks of the reduce jobs.
static_assert(SDY_ROWS == SDY_ROWS_HOST, "row blocks of scale_dy_rows");
__device__ __forceinline__ void multi_aux(int n_sdy, int n_red, int n_tp, int aux_wgs, int w, uint8_t *lds)
{
    struct { int n_sdy, n_red, n_tp, aux_wgs; } m{n_sdy, n_red, n_tp, aux_wgs};
    float *red = reinterpret_cast<float *>(lds);
    constexpr uint32_t SDY0 = offsetof(MultiArgs, sdy), RED0 = offsetof(MultiArgs, red), TP0 = offsetof(MultiArgs, tp);
    const int n_blk = m.n_sdy > 0 ? kernarg_load<int>(SDY0 + (uint32_t)((m.n_sdy - 1) * sizeof(ScaleDyJob) + offsetof(ScaleDyJob, blk_end))) : 0;
    const int n_chunk = m.n_red > 0 ? kernarg_load<int>(RED0 + (uint32_t)((m.n_red - 1) * sizeof(ReduceJob) + offsetof(ReduceJob, chunk_end))) : 0;
    const int n_tile = m.n_tp > 0 ? kernarg_load<int>(TP0 + (uint32_t)((m.n_tp - 1) * sizeof(TransposeJob) + offsetof(TransposeJob, tile_end))) : 0;
    for (int u = w; u < n_blk + n_chunk + n_tile; u += m.aux_wgs) {
        if (u >= n_blk + n_chunk) {
            const int x = u - n_blk - n_chunk;
            int j = 0, x0 = 0;
            for (int i = 0; i + 1 < m.n_tp; ++i) {
                const int e = kernarg_load<int>(TP0 + (uint32_t)(i * sizeof(TransposeJob) + offsetof(TransposeJob, tile_end)));
                if (x >= e) { j = i + 1; x0 = e; }
            }
            const TransposeJob J = kernarg_load<TransposeJob>(TP0 + (uint32_t)(j * sizeof(TransposeJob)));
            const int bts = J.Tp >> 6;
            transpose_pad_tile(J.src, J.T, J.C, J.dst, (x - x0) % bts, (x - x0) / bts, reinterpret_cast<uint16_t(*)[64 + 2]>(lds));
            __syncthreads();                                   // the LDS tile is reused by the next one
            continue;
        }
        if (u < n_blk) {
            int j = 0, b0 = 0;
            for (int i = 0; i + 1 < m.n_sdy; ++i) {
                const int e = kernarg_load<int>(SDY0 + (uint32_t)(i * sizeof(ScaleDyJob) + offsetof(ScaleDyJob, blk_end)));
                if (u >= e) { j = i + 1; b0 = e; }
            }
            const ScaleDyJob J = kernarg_load<ScaleDyJob>(SDY0 + (uint32_t)(j * sizeof(ScaleDyJob)));
            scale_dy_rows(J.dY, J.s0, J.ds, J.z0, nullptr, J.T, J.N, J.dYs, J.crow, u - b0, red);
            __syncthreads();                                   // `red` is reused by the next block
        } else {
            const int c = u - n_blk;
            int j = 0, c0 = 0;
            for (int i = 0; i + 1 < m.n_red; ++i) {
                const int e = kernarg_load<int>(RED0 + (uint32_t)(i * sizeof(ReduceJob) + offsetof(ReduceJob, chunk_end)));
                if (c >= e) { j = i + 1; c0 = e; }
            }
            const ReduceJob J = kernarg_load<ReduceJob>(RED0 + (uint32_t)(j * sizeof(ReduceJob)));
            reduce_partials_at(J.partial, J.ntiles, (size_t)J.n, (size_t)(c - c0) * 256 + threadIdx.x, J.out);
        }
    }
}

// Several per-channel contractions as four-wave tiles of one launch (see MultiArgs): workgroup -> (job, tile) by the
// jobs' running totals; the job's arguments come out of the argument block with scalar loads.
// GMODE < 0: per-channel jobs of any mode; GMODE = MODE_Y or MODE_DX: group-wise jobs, all of that mode (their
// scale gradient is the token contraction of peqa_dw.hip); GMODE_DX_ASIDE: group-wise dX jobs that all scale their
// activation fragments.
constexpr int GMODE_DX_ASIDE = 3;
static_assert(MODE_Y != 3 && MODE_DDS != 3 && MODE_DX != 3, "a value of its own");
template <int BITS, int GMODE>
__global__ __launch_bounds__(256, 2) void gemm_multi_kernel(MultiArgs m)
{
    extern __shared__ __align__(16) uint8_t lds[];
    int b = (int)blockIdx.x;
    if constexpr (GMODE != MODE_Y) {                           // a group-wise forward has no side work
        if (b >= m.aux_begin) {
            if (b < m.aux_begin + m.aux_wgs) {
                multi_aux(m.n_sdy, m.n_red, m.n_tp, m.aux_wgs, b - m.aux_begin, lds);
                return;
            }
            b -= m.aux_wgs;
        }
    }
    int j = 0, wg0 = 0;
#pragma unroll
    for (int i = 0; i < MULTI_MAX_JOBS - 1; ++i) {
        const int e = kernarg_load<int>((uint32_t)(i * sizeof(MultiJob) + offsetof(MultiJob, wg_end)));
        if (b >= e) { j = i + 1; wg0 = e; }
    }
    const GemmArgs a = kernarg_load<GemmArgs>((uint32_t)(j * sizeof(MultiJob) + offsetof(MultiJob, a)));
    if constexpr (GMODE == GMODE_DX_ASIDE) {
        gemm_tile<BITS, MODE_DX, true, 1, true>(a, b - wg0, lds);
    } else if constexpr (GMODE >= 0) {
        gemm_tile<BITS, GMODE, true, 1>(a, b - wg0, lds);
    } else {
        const int mode = kernarg_load<int>((uint32_t)(j * sizeof(MultiJob) + offsetof(MultiJob, mode)));
        if (mode == MODE_Y) gemm_tile<BITS, MODE_Y, false, 1>(a, b - wg0, lds);
        else if (mode == MODE_DDS) gemm_tile<BITS, MODE_DDS, false, 1>(a, b - wg0, lds);
        else gemm_tile<BITS, MODE_DX, false, 1>(a, b - wg0, lds);
    }
}

}  // namespace

// Contraction halves per workgroup.  Eight waves with two halves, one workgroup per compute unit, when a launch
// has at most one tile per compute unit (a lone four-wave workgroup leaves every SIMD a single wave, which
// measures 7-10 % slower); otherwise four waves with the whole range and two workgroups per compute unit
// (72 KB of LDS each), which fill the same four SIMDs with two waves each, need no exchange of partial sums,
// and hide one workgroup's ring fill and epilogue behind the other's loop.  The option gemm_waves = 4 or 8
// (peqa_set_option) forces one of them, for tests and comparisons.
static int halves_per_workgroup(int tiles, bool paired)
{
    if (paired) return 2;
    if (options().gemm_waves == 4) return 1;
    if (options().gemm_waves == 8) return 2;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    return tiles > cus ? 1 : 2;
}

bool gemm_four_waves(int tiles) { return halves_per_workgroup(tiles, false) == 1; }

template <int BITS, int MODE, bool GROUPED, int KW, bool ASCALE = false>
static hipError_t launch_one(const GemmArgs &a, hipStream_t stream)
{
    // dynamic LDS: the ring, plus the scale tables of the grouped forward / dX (twice as large for dX
    // when groups end inside a 128-feature run)
    const int lds_bytes = ring_bytes(KW) + (GROUPED && MODE != MODE_DDS ? (MODE == MODE_DX && (a.gsz & 127) ? 2 : 1) * tbl_bytes(KW) : 0);
    // the limit is a per-device attribute of every instantiation; raised to what a launch needs
    static int attr_bytes[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (attr_bytes[dev] < lds_bytes) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_kernel<BITS, MODE, GROUPED, KW, ASCALE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_bytes[dev] = lds_bytes;
    }
    const int pt = a.patch_t, pc = 32 / pt;
    const int patches = ((a.tiles_t + pt - 1) / pt) * ((a.tiles_c + pc - 1) / pc);
    const int grid = ((patches + 7) / 8) * 8 * 32;
    // grouped scale gradient: one pair of scale groups per workgroup along y
    const int gy = GROUPED && MODE == MODE_DDS ? (a.G + 1) / 2 : 1;
    // spare workgroups (see the kernel) exist in one instantiation only
    constexpr bool SPARE_TP = MODE == MODE_DX && GROUPED && KW == 1;
    if (!SPARE_TP && a.tp_blocks != 0) return hipErrorInvalidValue;
    const int spare_blocks = SPARE_TP ? a.tp_blocks : 0;
    hipLaunchKernelGGL((gemm_kernel<BITS, MODE, GROUPED, KW, ASCALE>), dim3(grid + spare_blocks, gy), dim3(256 * KW), lds_bytes,
                       stream, a);
    return hipGetLastError();
}

template <int BITS, int MODE, bool GROUPED>
static hipError_t launch_halves(const GemmArgs &a, hipStream_t stream)
{
    constexpr bool PAIRED = GROUPED && MODE == MODE_DDS;
    if constexpr (GROUPED && MODE == MODE_DX) {
        // scales on the activation side: the table is in that form, and only the four-wave tile reads it
        if (a.a_side) {
            if (a.gsz % 128 != 0 || halves_per_workgroup(a.tiles_t * a.tiles_c, false) != 1) return hipErrorInvalidValue;
            return launch_one<BITS, MODE, GROUPED, 1, true>(a, stream);
        }
    }
    if constexpr (!PAIRED) {
        if (halves_per_workgroup(a.tiles_t * a.tiles_c, false) == 1) return launch_one<BITS, MODE, GROUPED, 1>(a, stream);
    }
    return launch_one<BITS, MODE, GROUPED, 2>(a, stream);
}

template <int BITS, bool GROUPED>
static hipError_t dispatch_mode(int mode, const GemmArgs &a, hipStream_t stream)
{
    switch (mode) {
    case MODE_Y: return launch_halves<BITS, MODE_Y, GROUPED>(a, stream);
    case MODE_DDS: return launch_halves<BITS, MODE_DDS, GROUPED>(a, stream);
    default: return launch_halves<BITS, MODE_DX, GROUPED>(a, stream);
    }
}

static hipError_t dispatch(int bits, int mode, const GemmArgs &a, hipStream_t stream)
{
    const bool grouped = a.gsz > 0;
    if (bits == 4) return grouped ? dispatch_mode<4, true>(mode, a, stream) : dispatch_mode<4, false>(mode, a, stream);
    return grouped ? dispatch_mode<3, true>(mode, a, stream) : dispatch_mode<3, false>(mode, a, stream);
}

hipError_t launch_gemm(int bits, int mode, const GemmArgs &a_in, hipStream_t stream)
{
    GemmArgs a = a_in;
    a.patch_t = a.tiles_t >= 4 ? 4 : (a.tiles_t >= 2 ? 2 : 1);
    const int kid = mode == MODE_Y ? KID_GEMM_Y : (mode == MODE_DDS ? KID_GEMM_DDS : KID_GEMM_DX);
    trace_before(kid, stream);
    const hipError_t e = dispatch(bits, mode, a, stream);
    trace_after(kid, stream);
    return e;
}

// Scale gradient and dX of one per-channel layer in one launch (see gemm_bwd_pair_kernel).
template <int BITS>
static hipError_t launch_pair(const GemmArgs &a_dds, const GemmArgs &a_dx, hipStream_t stream)
{
    const int lds_bytes = ring_bytes(1);
    static int attr_bytes[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (attr_bytes[dev] < lds_bytes) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_bwd_pair_kernel<BITS>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_bytes[dev] = lds_bytes;
    }
    auto grid_of = [](const GemmArgs &a) {
        const int pt = a.patch_t, pc = 32 / pt;
        const int patches = ((a.tiles_t + pt - 1) / pt) * ((a.tiles_c + pc - 1) / pc);
        return ((patches + 7) / 8) * 8 * 32;               // a multiple of 8: both parts keep workgroup id % 8 = XCD
    };
    // the tiles that take longer go first: the short ones fill the last round better
    const int dx_first = a_dx.KC >= a_dds.KC;
    const int n_first = grid_of(dx_first ? a_dx : a_dds), n_second = grid_of(dx_first ? a_dds : a_dx);
    hipLaunchKernelGGL((gemm_bwd_pair_kernel<BITS>), dim3(n_first + n_second), dim3(256), lds_bytes, stream, a_dds, a_dx,
                       n_first, dx_first);
    return hipGetLastError();
}

int gemm_multi_wgs(int tiles_t, int tiles_c)
{
    const int pt = tiles_t >= 4 ? 4 : (tiles_t >= 2 ? 2 : 1), pc = 32 / pt;
    const int patches = ((tiles_t + pt - 1) / pt) * ((tiles_c + pc - 1) / pc);
    return ((patches + 7) / 8) * 8 * 32;
}

template <int BITS, int GMODE>
static hipError_t launch_multi(dim3 grid, int lds_bytes, const MultiArgs &m, hipStream_t stream)
{
    static int attr_bytes[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (attr_bytes[dev] < lds_bytes) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_multi_kernel<BITS, GMODE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_bytes[dev] = lds_bytes;
    }
    hipLaunchKernelGGL((gemm_multi_kernel<BITS, GMODE>), grid, dim3(256), lds_bytes, stream, m);
    return hipGetLastError();
}

hipError_t launch_gemm_multi(int bits, bool grouped, MultiArgs &m, hipStream_t stream)
{
    if (m.n_jobs < 0 || m.n_jobs > MULTI_MAX_JOBS || m.n_sdy < 0 || m.n_sdy > MULTI_MAX_JOBS || m.n_red < 0 ||
        m.n_red > MULTI_MAX_JOBS || m.n_tp < 0 || m.n_tp > 2 * MULTI_MAX_JOBS)
        return hipErrorInvalidValue;
    int total = 0, lds_bytes = ring_bytes(1);
    for (int j = 0; j < MULTI_MAX_JOBS; ++j) {
        if (j < m.n_jobs) {
            GemmArgs &a = m.job[j].a;
            if ((a.gsz > 0) != grouped || a.tp_blocks) return hipErrorInvalidValue;
            if (grouped && m.job[j].mode == MODE_DDS) return hipErrorInvalidValue;
            a.patch_t = a.tiles_t >= 4 ? 4 : (a.tiles_t >= 2 ? 2 : 1);
            total += gemm_multi_wgs(a.tiles_t, a.tiles_c);
            // group-wise: the scale tables behind the ring (twice as large for dX when groups end inside a 128-feature run)
            if (grouped) {
                const int need = ring_bytes(1) + (m.job[j].mode == MODE_DX && (a.gsz & 127) ? 2 : 1) * tbl_bytes(1);
                lds_bytes = need > lds_bytes ? need : lds_bytes;
            }
        } else {
            m.job[j] = m.job[m.n_jobs > 0 ? m.n_jobs - 1 : 0];
        }
        m.job[j].wg_end = total;
    }
    if ((m.aux_begin & 7) || (m.aux_wgs & 7) || m.aux_begin < 0 || m.aux_begin > total) return hipErrorInvalidValue;
    if (total + m.aux_wgs == 0) return hipSuccess;
    const int mode0 = m.n_jobs > 0 ? m.job[0].mode : MODE_DX;
    const bool a_side = grouped && m.n_jobs > 0 && m.job[0].a.a_side != 0;
    if (grouped) {
        for (int j = 0; j < m.n_jobs; ++j) {
            if (m.job[j].mode != mode0 || (m.job[j].a.a_side != 0) != a_side) return hipErrorInvalidValue;
            if (a_side && (mode0 != MODE_DX || m.job[j].a.gsz % 128 != 0)) return hipErrorInvalidValue;
        }
        if (mode0 == MODE_Y && m.aux_wgs != 0) return hipErrorInvalidValue;
    }
    const int kid = mode0 == MODE_Y ? KID_GEMM_MULTI_Y : (mode0 == MODE_DDS ? KID_GEMM_MULTI_DDS : KID_GEMM_MULTI_DX);
    trace_before(kid, stream);
    const dim3 grid(total + m.aux_wgs);
    hipError_t e;
    if (!grouped) e = bits == 4 ? launch_multi<4, -1>(grid, lds_bytes, m, stream) : launch_multi<3, -1>(grid, lds_bytes, m, stream);
    else if (mode0 == MODE_Y) e = bits == 4 ? launch_multi<4, MODE_Y>(grid, lds_bytes, m, stream) : launch_multi<3, MODE_Y>(grid, lds_bytes, m, stream);
    else if (a_side) e = bits == 4 ? launch_multi<4, GMODE_DX_ASIDE>(grid, lds_bytes, m, stream) : launch_multi<3, GMODE_DX_ASIDE>(grid, lds_bytes, m, stream);
    else e = bits == 4 ? launch_multi<4, MODE_DX>(grid, lds_bytes, m, stream) : launch_multi<3, MODE_DX>(grid, lds_bytes, m, stream);
    trace_after(kid, stream);
    return e;
}

hipError_t launch_gemm_bwd_pair(int bits, const GemmArgs &dds_in, const GemmArgs &dx_in, hipStream_t stream)
{
    GemmArgs a_dds = dds_in, a_dx = dx_in;
    if (a_dds.gsz > 0 || a_dx.gsz > 0 || a_dds.tp_blocks || a_dx.tp_blocks || a_dds.tiles_t != a_dx.tiles_t)
        return hipErrorInvalidValue;
    a_dds.patch_t = a_dx.patch_t = a_dds.tiles_t >= 4 ? 4 : (a_dds.tiles_t >= 2 ? 2 : 1);
    trace_before(KID_GEMM_BWD, stream);
    const hipError_t e = bits == 4 ? launch_pair<4>(a_dds, a_dx, stream) : launch_pair<3>(a_dds, a_dx, stream);
    trace_after(KID_GEMM_BWD, stream);
    return e;
}

}  // namespace peqa
