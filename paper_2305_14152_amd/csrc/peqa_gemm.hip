// Dense contractions of the PEQA linear layer on gfx950 MFMA (per-channel scales).
//
//   MODE_Y   : Y[t,i]    = s_i * sum_k X[t,k] (Q[i,k] - z_i)                (Eq. 2 forward)
//   MODE_DDS : part[i]   = sum_{t in tile} dY[t,i] * sum_k X[t,k] (Q[i,k] - z_i)
//                                                   (scale gradient, column-reduced epilogue)
//   MODE_DX  : dX[t,k]   = sum_i (dY[t,i] s_i) (Q[i,k] - z_i)                (chain rule on Eq. 2)
//
// One workgroup = 4 waves = a 128 (tokens) x 256 (output columns) tile.  Waves are laid out
// 2 (column halves) x 2 (halves of the contraction range): every wave owns a 128 x 128
// accumulator (8 x 8 MFMA 16x16x32 tiles, 256 fp32 registers) over its half of the
// contraction, so that a 2048 x 4096 output still fills all 256 CUs with one workgroup each.
// The two halves are summed through LDS in the epilogue (or, for MODE_DDS, after the
// column reduction, which is linear).
//
// Operand paths.  The activation operand (X, or the pre-scaled dY) goes global -> LDS ->
// registers (128 x 64 bf16 tiles, double buffered, 16-byte chunks XOR-swizzled by row).
// The weight operand never touches LDS: each lane loads the packed 8x8 code blocks it needs
// straight from global memory and unpacks them in registers into bf16 (16 + Q) fragments
// (peqa_device.h).  The contraction therefore runs on exact small integers; the offset 16,
// the zero-point and the scale are applied in the epilogue from row sums of the other
// operand:   sum_k X (Q - z) = sum_k X (16 + Q) - (16 + z) sum_k X.
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
constexpr int STAGE_BYTES = 2 * A_HALF_BYTES + 4 * B_WAVE_BYTES;   // 24 KB
constexpr int DMA_PER_ITER = 6;                            // DMA instructions per wave per iteration
constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES > 128 * 1024 ? NSTAGE * STAGE_BYTES : 128 * 1024;   // ring / epilogue exchange (128 KB)

// Global -> LDS DMA of 16 bytes per lane: lane l's bytes land at lds_dst + 16 l.  The source
// is sbase (uniform) + voff (per lane).  Issued from inline assembly so that the compiler does not
// serialise the ring with a conservative vmcnt(0); completion is tracked by hand with wait_vmcnt().
__device__ __forceinline__ void dma16(uint32_t voff, const void *sbase, uint32_t lds_dst)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(sbase), "s"(lds_dst) : "memory");
}
// Activation tiles sit in LDS as rows of 64 B (four 16-byte chunks).  Chunk j of row r is stored at
// position j ^ a_swizzle(r): with it, the 16-byte reads of 8 (16) consecutive rows at one logical
// chunk fall into 8 (16) different 16-byte bank groups of a 128 (256) byte LDS line.
__device__ __forceinline__ int a_swizzle(int row) { return ((row >> 1) & 3) ^ ((row >> 3) & 1); }

template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(std::integral_constant<int, N - 1>{});
    }
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    // gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14; other counters left open
    __builtin_amdgcn_s_waitcnt((N & 0xF) | (0x7 << 4) | (0xF << 8) | ((N >> 4) << 14));
}

template <int BITS, int MODE>
__global__ __launch_bounds__(256, 1) void gemm_kernel(GemmArgs a)
{
    extern __shared__ __align__(16) uint8_t lds[];
    constexpr int WPB = 2 * BITS;                          // words per 8x8 block
    constexpr bool ALONG_CH = (MODE == MODE_DX);           // contraction over output channels

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in an SGPR
    const int wn = wave & 1, wk = wave >> 1;
    const int c = lane & 15, q = lane >> 4;

    // workgroup -> tile.  Workgroup ids are dealt round-robin to the 8 XCDs and every CU holds one
    // workgroup, so the 32 ids {x, x + 8, ...} that run together on XCD x are given one patch of
    // patch_t x (32 / patch_t) neighbouring tiles: they share activation rows and weight columns
    // through that XCD's L2 instead of each pulling its own from the fabric.
    int tile_t, tile_c;
    {
        const int wg = blockIdx.x;
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
    const int khalf = KC >> 1;                             // both waves of a column half take KC/2
    const int kbeg = wk ? khalf : 0;
    const int nit = khalf / KSTEP;                         // loop iterations (>= 2: KC % 128 == 0)
    const int kblocks = a.K >> 3;                          // blocks per channel-row of blocks
    const uint32_t magic = kMagic;
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;

    // ---- activation tiles: global -> LDS by DMA, 16 wave-loads of 1 KB per iteration (4 per wave).
    // Wave-load m = 4 i + wave covers contraction half m / 8, rows 16 (m % 8) .. +16; lane s lands at
    // byte 16 s of that 1 KB, i.e. row s / 4, chunk position s % 4, and fetches the chunk that the
    // XOR swizzle assigns to that position.
    uint32_t a_voff[4];
    {
        const int row_l = lane >> 2, pos = lane & 3;
        const int chunk = pos ^ a_swizzle(row_l);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = 4 * i + wave;
            int row = (m & 7) * 16 + row_l;
            row = t0 + row < T ? row : T - 1 - t0;
            a_voff[i] = (uint32_t)row * (uint32_t)KC * 2u + (uint32_t)chunk * 16u;
        }
    }
    const uint8_t *a_base = reinterpret_cast<const uint8_t *>(a.A) + (size_t)t0 * KC * 2;

    // ---- packed weights: one 8x8 block per lane per iteration, also by DMA into the wave's own slot
    // along features: lane (c, q) owns channel block col0/8 + c and feature block 4 it + q
    // along channels: lane (c, q) owns feature block col0/8 + c and channel block 4 it + q
    const uint8_t *b_base;
    size_t b_step;                                         // bytes to advance per iteration
    uint32_t b_voff, b_voff2 = 0;
    int b_lane_off;                                        // where this lane's block sits in the wave's LDS slot
    if constexpr (!ALONG_CH) {
        b_base = reinterpret_cast<const uint8_t *>(a.packed + ((size_t)(col0 / 8) * kblocks + (kbeg >> 3)) * WPB);
        b_step = (size_t)4 * WPB * 4;
    } else {
        b_base = reinterpret_cast<const uint8_t *>(a.packed + ((size_t)(kbeg >> 3) * kblocks + col0 / 8) * WPB);
        b_step = (size_t)4 * kblocks * WPB * 4;
    }
    if constexpr (BITS == 4) {
        // two DMAs of 16 B per lane: the halves of the lane's own 32-byte block
        b_voff = (uint32_t)(ALONG_CH ? q * kblocks + c : c * kblocks + q) * 32u;
        b_lane_off = lane * 16;
    } else {
        // 24-byte blocks: the wave's 64 blocks form 16 runs of 96 B (along features) or 4 runs of
        // 384 B (along channels) = 96 chunks of 16 B, fetched as chunk `lane` and chunk `64 + lane`
        // and laid down in LDS in chunk order.
        constexpr int RUN = ALONG_CH ? 24 : 6;             // chunks per contiguous run
        const int x0 = lane, x1 = 64 + (lane & 31);
        b_voff = (uint32_t)(x0 / RUN) * (uint32_t)kblocks * 24u + (uint32_t)(x0 % RUN) * 16u;
        b_voff2 = (uint32_t)(x1 / RUN) * (uint32_t)kblocks * 24u + (uint32_t)(x1 % RUN) * 16u;
        b_lane_off = ALONG_CH ? q * 384 + c * 24 : c * 96 + q * 24;
    }
    if (!wave_on) { b_base = reinterpret_cast<const uint8_t *>(a.packed); b_step = 0; b_voff = lane * 32; b_voff2 = lane * 32; }

    auto issue = [&](int it, int stage) {
        const uint32_t sb = lds_base + stage * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = 4 * i + wave, h = m >> 3;
            dma16(a_voff[i], a_base + ((size_t)h * khalf + (size_t)it * KSTEP) * 2, sb + h * A_HALF_BYTES + (m & 7) * 1024);
        }
        const uint8_t *bp = b_base + (size_t)it * b_step;
        const uint32_t bb = sb + 2 * A_HALF_BYTES + wave * B_WAVE_BYTES;
        if constexpr (BITS == 4) {
            dma16(b_voff, bp, bb);
            dma16(b_voff, bp + 16, bb + 1024);
        } else {
            dma16(b_voff, bp, bb);
            dma16(b_voff2, bp, bb + 1024);      // lanes 32..63 repeat chunks 64..95 into the unused tail of the slot
        }
    };

    f32x4 acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // row = 16 rt + c and the swizzle only looks at row % 16
    const int a_read_off = wk * A_HALF_BYTES + c * 64 + ((q ^ a_swizzle(c)) << 4);
    const int b_read_off = 2 * A_HALF_BYTES + wave * B_WAVE_BYTES + b_lane_off;

    auto read_b = [&](int stage, uint32_t *bw) {
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

    auto read_a = [&](int stage, u32x4 *afrag, int rt) {
        afrag[rt] = *reinterpret_cast<const u32x4 *>(lds + stage * STAGE_BYTES + a_read_off + rt * 16 * 64);
    };

    // ---- prologue: queue NSTAGE - 1 stages, wait for the first two, fetch and unpack the operands
    // of step 0
    u32x4 bfrag[2][8], afrag[2][8];
#pragma unroll
    for (int sidx = 0; sidx < NSTAGE - 1; ++sidx) issue(sidx < nit ? sidx : nit - 1, sidx);
    wait_vmcnt<DMA_PER_ITER *(NSTAGE - 3)>();
    __syncthreads();
    {
        uint32_t bw[WPB];
        read_b(0, bw);
#pragma unroll
        for (int rt = 0; rt < 8; ++rt) read_a(0, afrag[0], rt);
        BlockUnpacker<BITS, ALONG_CH> up;
        up.prepare(bw);
        static_for<8>([&](auto i) { bfrag[0][i.value] = up.template frag<i.value>(magic); });
    }

    // ---- main loop.  A step is a 32-deep contraction: 64 MFMAs, one per accumulator.  When step
    // `it` starts, its operands are already in registers and stages it + 1 (next activations and
    // packed weights) are complete in LDS.  The step queues the DMA for step it + NSTAGE - 1 (the
    // tail re-fetches the last tile: harmless, and it keeps the DMA count per step constant so
    // that a fixed vmcnt tells when a stage has landed) and runs its MFMAs back to back, with the
    // unpacking of the next step's weights and the LDS reads of the next step's activations
    // spread between them.  Two steps per loop trip so that the register buffers are static.
    int cur = 0;                                           // LDS stage of the current step
    auto step = [&](int it, auto cur_c) {
        constexpr int CUR = decltype(cur_c)::value, NXT = CUR ^ 1;
        const int pre = it + NSTAGE - 1 < nit ? it + NSTAGE - 1 : nit - 1;
        const int nstage = cur + 1 == NSTAGE ? 0 : cur + 1;       // stage of step it + 1
        const int pstage = cur == 0 ? NSTAGE - 1 : cur - 1;       // stage of step it - 1 = of step it + NSTAGE - 1
        uint32_t bw[WPB];
        read_b(nstage, bw);
        read_a(nstage, afrag[NXT], 0);
#ifndef PEQA_EXP_NO_DMA
        issue(pre, pstage);
#endif
        BlockUnpacker<BITS, ALONG_CH> up;
        static_for<8>([&](auto rt_c) {
            constexpr int rt = rt_c.value;
            if constexpr (rt == 0) up.prepare(bw);
            if constexpr (rt < 7) read_a(nstage, afrag[NXT], rt + 1);   // last LDS read one group before the barrier
            static_for<8>([&](auto ct_c) {
                constexpr int ct = ct_c.value;
#ifndef PEQA_EXP_NO_MFMA
                mfma16_acc(acc[rt][ct], afrag[CUR][rt], bfrag[CUR][ct]);
#endif
                // one register of the next step's fragment rt in the shadow of every other MFMA
#ifndef PEQA_EXP_NO_UNPACK
                if constexpr (ct & 1) bfrag[NXT][rt][ct >> 1] = up.template frag_reg<rt, (ct >> 1)>(magic);
#endif
            });
        });
        // Own DMA for the stage after next has landed; the barrier makes every wave's part visible.
        // No wait on LDS reads is needed here: what this step read is overwritten two steps later.
        wait_vmcnt<DMA_PER_ITER *(NSTAGE - 3)>();
        bare_barrier();
        cur = nstage;
    };
    for (int it = 0; it < nit; it += 2) {                  // nit is even: KC % 128 == 0
        step(it, std::integral_constant<int, 0>{});
        step(it + 1, std::integral_constant<int, 1>{});
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
            float zoff[8];
            {
                const uint8_t *zp = a.z0 + col0 + 8 * c;
                const u32x2 zz = *reinterpret_cast<const u32x2 *>(zp);
#pragma unroll
                for (int ct = 0; ct < 8; ++ct)
                    zoff[ct] = kCodeOffset + (float)((zz[ct >> 2] >> (8 * (ct & 3))) & 0xFFu);
            }
#pragma unroll
            for (int rt = 0; rt < 8; ++rt) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int t = t0 + rt * 16 + 4 * q + j;
                    if (t < T) {
                        const u32x4 dy = *reinterpret_cast<const u32x4 *>(a.dY + (size_t)t * a.C + col0 + 8 * c);
                        const float r = a.rs[2 * t + wk];
#pragma unroll
                        for (int ct = 0; ct < 8; ++ct) {
                            const float d = (ct & 1) ? bf16_hi(dy[ct >> 1]) : bf16_lo(dy[ct >> 1]);
                            colsum[ct] += d * (acc[rt][ct][j] - zoff[ct] * r);
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) {
            colsum[ct] += __shfl_xor(colsum[ct], 16);
            colsum[ct] += __shfl_xor(colsum[ct], 32);
        }
        float *red = reinterpret_cast<float *>(lds);           // [4 waves][128]
        if (q == 0) {
#pragma unroll
            for (int ct = 0; ct < 8; ++ct) red[wave * 128 + 8 * c + ct] = colsum[ct];
        }
        __syncthreads();
        {
            const int w2 = tid >> 7, col = tid & 127;          // column half, column in half
            const int n = tile_c * TILE_C + tid;
            if (n < a.C) a.partial[(size_t)tile_t * a.C + n] = red[w2 * 128 + col] + red[(2 + w2) * 128 + col];
        }
    } else {
        // sum the two contraction halves: wave wk keeps row tiles [4 wk, 4 wk + 4) and sends the others
        f32x4 *xch = reinterpret_cast<f32x4 *>(lds);           // [4 waves][32 tiles][64 lanes]
        auto finish = [&](auto keep_c) {
            constexpr int KEEP = decltype(keep_c)::value;      // first row tile this wave keeps
            constexpr int SEND = 4 - KEEP;
            {
                f32x4 *mine = xch + (size_t)wave * 32 * 64 + lane;
#pragma unroll
                for (int rtl = 0; rtl < 4; ++rtl)
#pragma unroll
                    for (int ct = 0; ct < 8; ++ct) mine[(rtl * 8 + ct) * 64] = acc[SEND + rtl][ct];
            }
            __syncthreads();
            if (!wave_on) return;
            const f32x4 *theirs = xch + (size_t)(wave ^ 2) * 32 * 64 + lane;
            float sc[8], zoff[8];
            if constexpr (MODE == MODE_Y) {
                const float *sp = a.s0 + col0 + 8 * c;
                const u32x2 zz = *reinterpret_cast<const u32x2 *>(a.z0 + col0 + 8 * c);
#pragma unroll
                for (int ct = 0; ct < 8; ++ct) {
                    sc[ct] = a.ds ? sp[ct] + a.ds[col0 + 8 * c + ct] : sp[ct];
                    zoff[ct] = kCodeOffset + (float)((zz[ct >> 2] >> (8 * (ct & 3))) & 0xFFu);
                }
            }
#pragma unroll
            for (int rtl = 0; rtl < 4; ++rtl) {
                f32x4 sum[8];
#pragma unroll
                for (int ct = 0; ct < 8; ++ct) sum[ct] = acc[KEEP + rtl][ct] + theirs[(rtl * 8 + ct) * 64];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int t = t0 + (KEEP + rtl) * 16 + 4 * q + j;
                    if (t < T) {
                        float v[8];
                        if constexpr (MODE == MODE_Y) {
                            const float r = a.rs[2 * t] + a.rs[2 * t + 1];
#pragma unroll
                            for (int ct = 0; ct < 8; ++ct) v[ct] = sc[ct] * (sum[ct][j] - zoff[ct] * r);
                        } else {
                            const float cc = a.crow[t];
#pragma unroll
                            for (int ct = 0; ct < 8; ++ct) v[ct] = sum[ct][j] - cc;
                        }
                        u32x4 o;
#pragma unroll
                        for (int p = 0; p < 4; ++p) o[p] = pack_bf16x2(v[2 * p], v[2 * p + 1]);
                        *reinterpret_cast<u32x4 *>(a.out + (size_t)t * a.C + col0 + 8 * c) = o;
                    }
                }
            }
        };
        if (wk == 0) finish(std::integral_constant<int, 0>{});
        else finish(std::integral_constant<int, 4>{});
    }
}

}  // namespace

int gemm_lds_bytes() { return LDS_BYTES; }

template <int BITS, int MODE>
static hipError_t launch_one(const GemmArgs &a, hipStream_t stream)
{
    static bool attr_done = false;                          // per instantiation
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_kernel<BITS, MODE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    const int pt = a.patch_t, pc = 32 / pt;
    const int patches = ((a.tiles_t + pt - 1) / pt) * ((a.tiles_c + pc - 1) / pc);
    const int grid = ((patches + 7) / 8) * 8 * 32;
    hipLaunchKernelGGL((gemm_kernel<BITS, MODE>), dim3(grid), dim3(256), LDS_BYTES, stream, a);
    return hipGetLastError();
}

static hipError_t dispatch(int bits, int mode, const GemmArgs &a, hipStream_t stream)
{
    if (bits == 4) {
        switch (mode) {
        case MODE_Y: return launch_one<4, MODE_Y>(a, stream);
        case MODE_DDS: return launch_one<4, MODE_DDS>(a, stream);
        default: return launch_one<4, MODE_DX>(a, stream);
        }
    }
    switch (mode) {
    case MODE_Y: return launch_one<3, MODE_Y>(a, stream);
    case MODE_DDS: return launch_one<3, MODE_DDS>(a, stream);
    default: return launch_one<3, MODE_DX>(a, stream);
    }
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

}  // namespace peqa
