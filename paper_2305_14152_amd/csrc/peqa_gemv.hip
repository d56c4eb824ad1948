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
// Grid: (N / 128 channel tiles) x (S feature slices).  A slice is a run of chunks (a chunk = one
// scale group, or 128 features); the 4 waves of a workgroup take consecutive quarters of it and are
// summed through LDS at the end.  S > 1 leaves fp32 partials [S, T, N] in the workspace for
// gemv_finish_kernel to add up in a fixed order.
//
// A wave moves its operands in rounds of 64 features (two MFMA steps): the packed blocks of its 16
// channel-block rows and the matching 128 bytes of each of the 16 token rows, by global -> LDS DMA
// into a private double buffer, from which each lane reads back its own blocks and activation
// fragments.  The LDS placement is chosen for conflict-free read-back: at 4 bits every lane's two
// 16-byte block halves sit at 16 * lane of two 1 KB planes per step; at 3 bits the 96 16-byte
// chunks of a step lie in address order (rows of 96 B).  No barrier is involved: a wave waits for
// its own DMA only.
#include <type_traits>

#include "peqa_device.h"
#include "peqa_kernels.h"

namespace peqa {

namespace {

constexpr int GV_WAVES = 4;
constexpr int GV_MAX_PER = 8;        // most chunks per slice of a group-wise layer (bounds the scale tile in LDS)
constexpr int GV_B_BYTES = 4096;     // packed blocks of one round of one wave (4 KB at 4 bits, 3 KB at 3 bits)
constexpr int GV_ROUND_BYTES = GV_B_BYTES + 2048;   // + 16 token rows x 128 B

struct ScaleZero { float s, zoff; };  // s0 + ds and 16 + z0

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

template <int BITS>
__global__ __launch_bounds__(GV_WAVES * 64, 2) void gemv_kernel(GemvArgs a)
{
    // [wave][2 rounds][6 KB]; reused as [wave][column tile][row][lane] fp32 (32 KB) for the final sum
    __shared__ __align__(16) uint8_t stage[GV_WAVES * 2 * GV_ROUND_BYTES];
    __shared__ __align__(8) ScaleZero sz[128][GV_MAX_PER];       // [channel][chunk of the slice], 8 KB
    constexpr int WPB = 2 * BITS;
    constexpr int NDMA_B = 2 * 64 * WPB * 4 / 1024;               // 1 KB DMAs for the blocks of a round: 4 / 3
    constexpr int NDMA = NDMA_B + 2;                              // + 2 for the token rows
    const int tid = threadIdx.x, lane = tid & 63;
#ifdef PEQA_EXP_GVTIMING
    uint64_t tk[5];
    tk[0] = __builtin_amdgcn_s_memrealtime();
#endif
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, q = lane >> 4;
    const int n0 = blockIdx.x * 128;
    const int K = a.K, G = a.G;
    const int chunk_rounds = a.chunk >> 6;                        // 64-feature rounds per chunk
    // this workgroup's chunks [cbeg, cend); wave w takes a contiguous quarter of them
    const int nchunks = K / a.chunk;
    const int per = (nchunks + a.S - 1) / a.S;
    const int cbeg = blockIdx.y * per;
    const int cend = cbeg + per < nchunks ? cbeg + per : nchunks;
    const int pw = (cend - cbeg + GV_WAVES - 1) / GV_WAVES;
    const int wc0 = cbeg + wave * pw < cend ? cbeg + wave * pw : cend;
    const int wc1 = wc0 + pw < cend ? wc0 + pw : cend;
    const int k0 = wc0 * a.chunk;                                 // first feature of this wave
    const int nrounds = (wc1 - wc0) * chunk_rounds;               // 64-feature rounds of this wave

    const uint32_t magic = kMagic;
    const u32x4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
    // the wave's tiles (128 channels x 32 features, TILE bytes each) are contiguous along the features
    constexpr uint32_t TILE = 64 * WPB * 4;
    const uint8_t *bbase = reinterpret_cast<const uint8_t *>(a.packed) +
                           ((size_t)blockIdx.x * (K >> 5) + (k0 >> 5)) * TILE;
    const uint8_t *xbase = reinterpret_cast<const uint8_t *>(a.X + k0);
    const uint32_t lds_stage = (uint32_t)(uintptr_t)stage + wave * 2 * GV_ROUND_BYTES;
    uint32_t b_voff[NDMA_B], x_voff[2];
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
    for (int i = 0; i < 2; ++i) {
        const int x = 64 * i + lane;                              // chunk x: token row x / 8, 16 bytes x % 8
        const int t = (x >> 3) < a.T ? (x >> 3) : a.T - 1;        // rows beyond T repeat the last one (never stored)
        x_voff[i] = (uint32_t)t * (uint32_t)K * 2u + (uint32_t)(x & 7) * 16u;
    }
    auto issue_round = [&](int r) {
        const uint32_t dst = lds_stage + (r & 1) * GV_ROUND_BYTES;
        const uint8_t *bsrc = bbase + (size_t)r * 2 * TILE;       // two tiles per round
#pragma unroll
        for (int i = 0; i < NDMA_B; ++i) gv_dma16(b_voff[i], bsrc, dst + i * 1024);
        const uint8_t *xsrc = xbase + (size_t)r * 128;
        gv_dma16(x_voff[0], xsrc, dst + GV_B_BYTES);
        gv_dma16(x_voff[1], xsrc, dst + GV_B_BYTES + 1024);
    };
    if (nrounds > 0) issue_round(0);
    if (nrounds > 1) issue_round(1);
#ifdef PEQA_EXP_GVTIMING
    tk[1] = __builtin_amdgcn_s_memrealtime();
#endif

    // scale / zero-point tile of the slice: [128 channels][chunks], or one column for per-channel
    // layers.  All its loads are issued together (indices clamped instead of branching, so that
    // the compiler batches them behind a single wait); that wait also covers the two rounds above,
    // which every wave needs next anyway.
    const int cols = a.grouped ? cend - cbeg : 1;
    {
        float ts[GV_MAX_PER / 2], td[GV_MAX_PER / 2];
        uint8_t tz[GV_MAX_PER / 2];
#pragma unroll
        for (int i = 0; i < GV_MAX_PER / 2; ++i) {
            const int idx = tid + i * GV_WAVES * 64;
            const int ch = idx < 128 * cols ? idx / cols : 0, j = idx < 128 * cols ? idx - ch * cols : 0;
            const size_t si = (size_t)(n0 + ch) * G + (a.grouped ? cbeg + j : 0);
            ts[i] = a.s0[si];
            tz[i] = a.z0[si];
            td[i] = a.ds ? a.ds[si] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < GV_MAX_PER / 2; ++i) {
            const int idx = tid + i * GV_WAVES * 64;
            if (idx < 128 * cols) {
                const int ch = idx / cols, j = idx - ch * cols;
                sz[ch][j] = ScaleZero{ts[i] + td[i], kCodeOffset + (float)tz[i]};
            }
        }
    }
    __syncthreads();
#ifdef PEQA_EXP_GVTIMING
    tk[2] = __builtin_amdgcn_s_memrealtime();
#endif

    f32x4 y[8], acc[8], accrs = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) { y[ct] = f32x4{0.f, 0.f, 0.f, 0.f}; acc[ct] = f32x4{0.f, 0.f, 0.f, 0.f}; }

    // this lane's block of step 0 within a round (step 1: + 2048 at 4 bits, + 1536 at 3 bits)
    const int b_off = BITS == 4 ? lane * 16 : c * 96 + q * 24;
    const int x_off = GV_B_BYTES + c * 128 + q * 16;              // this lane's activation fragment of step 0
    auto compute_round = [&](int r, auto buf_c) {
        constexpr int BUF = decltype(buf_c)::value;
        // rounds r and (if any) r + 1 are in flight: wait for r only
#ifndef PEQA_EXP_NO_WAIT
        if (r + 1 < nrounds) gv_wait_vmcnt<NDMA>(); else gv_wait_vmcnt<0>();
#endif
        const uint8_t *st = stage + (wave * 2 + BUF) * GV_ROUND_BYTES;
#ifdef PEQA_EXP_NO_COMPUTE
        if (a.T > 99)
#endif
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            uint32_t bw[WPB];
            if constexpr (BITS == 4) {
                const u32x4 v0 = *reinterpret_cast<const u32x4 *>(st + b_off + s2 * 2048);
                const u32x4 v1 = *reinterpret_cast<const u32x4 *>(st + b_off + s2 * 2048 + 1024);
#pragma unroll
                for (int i = 0; i < 4; ++i) { bw[i] = v0[i]; bw[4 + i] = v1[i]; }
            } else {
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    const u32x2 v = *reinterpret_cast<const u32x2 *>(st + b_off + s2 * 1536 + 8 * i);
                    bw[2 * i] = v[0];
                    bw[2 * i + 1] = v[1];
                }
            }
            const u32x4 af = *reinterpret_cast<const u32x4 *>(st + x_off + s2 * 64);
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
        // this buffer is free again (its LDS reads have returned: the MFMAs consumed them): refill it
        if (r + 2 < nrounds) issue_round(r + 2);
    };
    auto flush_if_chunk_end = [&](int r) {
        if ((r + 1) % chunk_rounds == 0) {
            // end of a chunk: fold offset, zero-point and scale of its group, restart the sums
            const int j = a.grouped ? wc0 - cbeg + (r + 1) / chunk_rounds - 1 : 0;
#pragma unroll
            for (int ct = 0; ct < 8; ++ct) {
                const ScaleZero v = sz[8 * c + ct][j];
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) y[ct][jj] += v.s * (acc[ct][jj] - v.zoff * accrs[jj]);
                acc[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            accrs = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    };

    if (nrounds > 0) compute_round(0, std::integral_constant<int, 0>{});
    if (nrounds > 0) flush_if_chunk_end(0);
    for (int r = 1; r < nrounds; r += 2) {
        compute_round(r, std::integral_constant<int, 1>{});
        flush_if_chunk_end(r);
        if (r + 1 < nrounds) {
            compute_round(r + 1, std::integral_constant<int, 0>{});
            flush_if_chunk_end(r + 1);
        }
    }

#ifdef PEQA_EXP_GVTIMING
    asm volatile("" :: "v"(y[0][0]), "v"(y[7][3]));
    tk[3] = __builtin_amdgcn_s_memrealtime();
#endif
    // ---- sum the waves, then write Y (S = 1) or this slice's partial
    __syncthreads();                                              // everyone is done with the stage buffers
    float *red = reinterpret_cast<float *>(stage);                // [wave][column tile][row in lane][lane], 32 KB
#pragma unroll
    for (int ct = 0; ct < 8; ++ct)
#pragma unroll
        for (int j = 0; j < 4; ++j) red[((wave * 8 + ct) * 4 + j) * 64 + lane] = y[ct][j];
    __syncthreads();
    // thread (wave, lane) finishes column tiles 2 wave, 2 wave + 1 of lane's rows/column
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int ct = 2 * wave + i;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float v = 0.f;
#pragma unroll
            for (int w = 0; w < GV_WAVES; ++w) v += red[((w * 8 + ct) * 4 + j) * 64 + lane];
            const int t = 4 * q + j, n = n0 + 8 * c + ct;
            if (t < a.T) {
                if (a.S == 1) a.Y[(size_t)t * a.N + n] = (uint16_t)float_to_bf16_bits(v);
                else a.partial[((size_t)blockIdx.y * a.T + t) * a.N + n] = v;
            }
        }
    }
#ifdef PEQA_EXP_GVTIMING
    tk[4] = __builtin_amdgcn_s_memrealtime();
    if (tid == 0) {
        uint64_t *d = reinterpret_cast<uint64_t *>(a.partial + (size_t)a.S * a.T * a.N) + (size_t)(blockIdx.y * gridDim.x + blockIdx.x) * 8;
        for (int i = 0; i < 5; ++i) d[i] = tk[i];
    }
#endif
}

// Y[t,n] = bf16( partial[0][t,n] + partial[1][t,n] + ... ), fixed order.
__global__ __launch_bounds__(256) void gemv_finish_kernel(const float *__restrict__ partial, int S, size_t tn,
                                                           uint16_t *__restrict__ Y)
{
    const size_t j = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= tn) return;
    float v = 0.f;
    for (int s = 0; s < S; ++s) v += partial[(size_t)s * tn + j];
    Y[j] = (uint16_t)float_to_bf16_bits(v);
}

}  // namespace

int gemv_slices(int N, int K, int T, int chunk, int grouped)
{
    // enough workgroups to cover the chip a few times over, every wave at least one chunk,
    // and partials kept small next to the weight bytes
    const int tiles = N / 128, nchunks = K / chunk;
    int S = (512 + tiles - 1) / tiles;
    const int by_chunks = nchunks / GV_WAVES > 0 ? nchunks / GV_WAVES : 1;
    if (S > by_chunks) S = by_chunks;
    const int by_bytes = T > 4 ? 6 : 16;
    if (S > by_bytes) S = by_bytes;
    if (S < 1) S = 1;
    // the scale tile in LDS holds at most GV_MAX_PER chunks per slice of a group-wise layer
    const int min_S = grouped ? (nchunks + GV_MAX_PER - 1) / GV_MAX_PER : 1;
    if (S < min_S) S = min_S;
    return S;
}

hipError_t launch_gemv(int bits, const GemvArgs &a, hipStream_t stream)
{
    trace_before(KID_GEMV, stream);
    const dim3 grid(a.N / 128, a.S);
    if (bits == 4) hipLaunchKernelGGL(gemv_kernel<4>, grid, dim3(GV_WAVES * 64), 0, stream, a);
    else hipLaunchKernelGGL(gemv_kernel<3>, grid, dim3(GV_WAVES * 64), 0, stream, a);
    trace_after(KID_GEMV, stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.S == 1) return e;
    trace_before(KID_GEMV_FINISH, stream);
    const size_t tn = (size_t)a.T * a.N;
    hipLaunchKernelGGL(gemv_finish_kernel, dim3((unsigned)((tn + 255) / 256)), dim3(256), 0, stream, a.partial, a.S, tn,
                       a.Y);
    trace_after(KID_GEMV_FINISH, stream);
    return hipGetLastError();
}

}  // namespace peqa
