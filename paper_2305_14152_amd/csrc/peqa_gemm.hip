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
#include "peqa_device.h"
#include "peqa_kernels.h"

namespace peqa {

namespace {

constexpr int TILE_T = 128;
constexpr int TILE_C = 256;
constexpr int KSTEP = 64;
constexpr int A_TILE_BYTES = TILE_T * KSTEP * 2;          // 16 KB
constexpr int LDS_BYTES = 128 * 1024;                      // A stages (64 KB) / epilogue exchange (128 KB)

template <int BITS, int MODE>
__global__ __launch_bounds__(256, 1) void gemm_kernel(GemmArgs a)
{
    extern __shared__ __align__(16) uint8_t lds[];
    constexpr int WPB = 2 * BITS;                          // words per 8x8 block
    constexpr bool ALONG_CH = (MODE == MODE_DX);           // contraction over output channels

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave & 1, wk = wave >> 1;
    const int c = lane & 15, q = lane >> 4;

    // workgroup -> tile.  Consecutive workgroup ids land on different XCDs; giving each XCD a
    // contiguous run of column tiles keeps a weight slab in one L2.
    const int tiles_c = a.tiles_c, tiles_t = a.tiles_t;
    int wg = blockIdx.x;
    {
        const int total = tiles_c * tiles_t;
        const int per_xcd = (total + 7) / 8;
        const int xcd = wg & 7, idx = wg >> 3;
        const int remapped = xcd * per_xcd + idx;
        // only use the remap when it is a bijection of [0, total)
        if ((total & 7) == 0) wg = remapped;
    }
    const int tile_t = wg % tiles_t, tile_c = wg / tiles_t;

    const int t0 = tile_t * TILE_T;
    const int col0 = tile_c * TILE_C + wn * 128;           // first output column of this wave
    const bool wave_on = col0 < a.C;
    const int T = a.T, KC = a.KC;
    const int kbeg = wk ? a.ksplit : 0;
    const int nsteps0 = a.ksplit / KSTEP, nsteps1 = (KC - a.ksplit) / KSTEP;
    const int nsteps_mine = wk ? nsteps1 : nsteps0;
    const int nsteps = nsteps0 > nsteps1 ? nsteps0 : nsteps1;
    const int kblocks = a.K >> 3;                          // blocks per channel-row of blocks

    const uint32_t magic = kMagic;

    // ---- activation tile loads: 8 chunks of 16 B per thread per step (4 per contraction half)
    const int a_row = tid >> 3, a_c8 = tid & 7;
    const uint16_t *a_src[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int t = t0 + j * 32 + a_row;
        t = t < T ? t : T - 1;
        a_src[j] = a.A + (size_t)t * KC + a_c8 * 8;
    }
    const int a_lds_off = a_row * 128 + ((a_c8 ^ (a_row & 7)) << 4);

    // ---- packed weight loads
    // along features: lane (c, q) owns channel block col0/8 + c and feature blocks 2q, 2q+1 of the step
    // along channels: lane (c, q) owns feature block col0/8 + c and channel blocks 2q, 2q+1 of the step
    const uint32_t *b_src;
    size_t b_step;                                         // words to advance per contraction step
    size_t b_second;                                       // offset of the lane's second block
    if constexpr (!ALONG_CH) {
        b_src = a.packed + ((size_t)(col0 / 8 + c) * kblocks + (kbeg >> 3) + 2 * q) * WPB;
        b_step = (size_t)8 * WPB;
        b_second = WPB;
    } else {
        b_src = a.packed + ((size_t)((kbeg >> 3) + 2 * q) * kblocks + (col0 / 8 + c)) * WPB;
        b_step = (size_t)8 * kblocks * WPB;
        b_second = (size_t)kblocks * WPB;
    }

    u32x4 areg[8];
    uint32_t breg[2][2 * WPB];

    auto load_a = [&](int ks) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int ns = h ? nsteps1 : nsteps0;
            const int kb = (h ? a.ksplit : 0) + ks * KSTEP;
            if (ks < ns) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    areg[h * 4 + j] = *reinterpret_cast<const u32x4 *>(a_src[j] + kb);
            }
        }
    };
    auto store_a = [&](int ks, int stage) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int ns = h ? nsteps1 : nsteps0;
            if (ks < ns) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    *reinterpret_cast<u32x4 *>(lds + (h * 2 + stage) * A_TILE_BYTES + j * 32 * 128 + a_lds_off) =
                        areg[h * 4 + j];
            }
        }
    };
    auto load_b = [&](int ks, int buf) {
        if (wave_on && ks < nsteps_mine) {
            const uint32_t *p = b_src + (size_t)ks * b_step;
#pragma unroll
            for (int blk = 0; blk < 2; ++blk) {
                const uint32_t *pb = p + blk * b_second;
                if constexpr (BITS == 4) {
                    const u32x4 v0 = *reinterpret_cast<const u32x4 *>(pb);
                    const u32x4 v1 = *reinterpret_cast<const u32x4 *>(pb + 4);
#pragma unroll
                    for (int i = 0; i < 4; ++i) { breg[buf][blk * 8 + i] = v0[i]; breg[buf][blk * 8 + 4 + i] = v1[i]; }
                } else {
#pragma unroll
                    for (int i = 0; i < 3; ++i) {
                        const u32x2 v = *reinterpret_cast<const u32x2 *>(pb + 2 * i);
                        breg[buf][blk * 6 + 2 * i] = v[0];
                        breg[buf][blk * 6 + 2 * i + 1] = v[1];
                    }
                }
            }
        }
    };

    f32x4 acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // ---- prologue
    load_a(0);
    load_b(0, 0);
    store_a(0, 0);
    __syncthreads();

    const int a_read_base = wk * 2 * A_TILE_BYTES + c * 128;   // row = 16 rt + c; row & 7 = c & 7
    const int csw = c & 7;

    for (int ks = 0; ks < nsteps; ++ks) {
        const int stage = ks & 1;
        load_a(ks + 1);
        load_b(ks + 1, stage ^ 1);
        if (wave_on && ks < nsteps_mine) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                u32x4 bfrag[8];
                if constexpr (!ALONG_CH) unpack_along_features<BITS>(&breg[stage][j * WPB], bfrag, magic);
                else unpack_along_channels<BITS>(&breg[stage][j * WPB], bfrag, magic);
                const int chunk = ((2 * q + j) ^ csw) << 4;
#pragma unroll
                for (int rt = 0; rt < 8; ++rt) {
                    const u32x4 afrag = *reinterpret_cast<const u32x4 *>(
                        lds + a_read_base + stage * A_TILE_BYTES + rt * 16 * 128 + chunk);
#pragma unroll
                    for (int ct = 0; ct < 8; ++ct) acc[rt][ct] = mfma16(afrag, bfrag[ct], acc[rt][ct]);
                }
            }
        }
        store_a(ks + 1, stage ^ 1);
        __syncthreads();
    }

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
        {
            f32x4 *mine = xch + (size_t)wave * 32 * 64 + lane;
#pragma unroll
            for (int rtl = 0; rtl < 4; ++rtl)
#pragma unroll
                for (int ct = 0; ct < 8; ++ct) {
                    // send the half I do not keep
                    mine[(rtl * 8 + ct) * 64] = wk ? acc[rtl][ct] : acc[4 + rtl][ct];
                }
        }
        __syncthreads();
        if (wave_on) {
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
                for (int ct = 0; ct < 8; ++ct) {
                    const f32x4 o = theirs[(rtl * 8 + ct) * 64];
                    const f32x4 m = wk ? acc[4 + rtl][ct] : acc[rtl][ct];
                    sum[ct] = m + o;
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int t = t0 + (4 * wk + rtl) * 16 + 4 * q + j;
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
        }
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
    const int total = a.tiles_c * a.tiles_t;
    hipLaunchKernelGGL((gemm_kernel<BITS, MODE>), dim3(total), dim3(256), LDS_BYTES, stream, a);
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

hipError_t launch_gemm(int bits, int mode, const GemmArgs &a, hipStream_t stream)
{
    const int kid = mode == MODE_Y ? KID_GEMM_Y : (mode == MODE_DDS ? KID_GEMM_DDS : KID_GEMM_DX);
    trace_before(kid, stream);
    const hipError_t e = dispatch(bits, mode, a, stream);
    trace_after(kid, stream);
    return e;
}

}  // namespace peqa
