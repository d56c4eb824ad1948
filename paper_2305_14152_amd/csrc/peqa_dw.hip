// Scale gradient of group-wise layers by the second route of the chain rule on Eq. 2:
//
//   dW[i,k]   = sum_t dY[t,i] X[t,k]                         (plain bf16 contraction over tokens)
//   d_ds[i,g] = sum_{k in g} dW[i,k] (Q[i,k] - z[i,g])       (codes applied once, in the epilogue)
//
// The first route (contract X with the codes group by group, then reduce over tokens) restarts its
// accumulators at every scale group: with 128 features per group a workgroup gets four steps of
// contraction between a ring fill and an epilogue.  Here the contraction runs over all tokens without a
// restart, no code is unpacked inside the loop, and the groups only appear in the epilogue.
//
// Both operands are needed with the token index contiguous, so X and dY are first transposed
// (transpose_pad_kernel) into step-major arrays [Tp / 32][rows][32] (rows = K or N, Tp = T rounded up to
// 64, zero-filled): the 64 bytes a row contributes to one 32-token step of the contraction sit next to
// those of its neighbour rows, so a tile of 256 rows is 16 contiguous KB per step.  (With plain [rows][Tp]
// arrays every 64-byte piece is half a cache line on its own, 2 Tp bytes from the next, and the loop
// is bound by the request rate of the L2: measured 1.5 us per step against 0.5 us of matrix work.)
//
// dw_kernel: one workgroup = a 256 (features) x 256 (channels) tile of dW, as 8 waves (4 along the features x
// 2 along the channels, two per SIMD) of 64 x 128 accumulators each (4 x 8 MFMA 16x16x32 tiles in 128 AGPRs);
// the template also builds 4 waves of 128 x 128 (one per SIMD), which measured slower (282 against 223 us on
// the 13B shapes: with one wave per SIMD nothing runs behind a wave's waits).  Both operands come from LDS.
// A wave's features are 64-feature chunks, the unit in which the epilogue reports (every group is a whole
// number of chunks).  Operands go global -> LDS by DMA into a ring of 4 stages of 32 KB (one 32-token step:
// 256 + 256 rows of 64 B, XOR-swizzled as in the other contraction kernel); fragments for step it + 1 are read
// from LDS while step it's matrix instructions run.  The epilogue takes each lane's codes from a copy of the tile's
// packed words that one of the ring's spare stages brought into LDS (see issue_one), at word positions and shifts
// worked out once per lane, forms sum dW Q - z sum dW over each chunk with two shuffles, and writes pc[i, chunk];
// chunk_reduce_kernel adds the chunks of every group in order.
// Where the time of a tile goes at T = 2048 (64 steps; timestamps per workgroup on the 13B shapes): 2.6 us from its
// start to its first fragments, 47-53 us in the loop (0.75-0.85 us per step against 0.49 us of matrix instructions:
// timing builds without the loop's DMAs, without its fragment reads, and without both ran the launch in 0.80, 0.92
// and 0.78 of its time, so with one workgroup per compute unit and a barrier per step about three quarters of the
// loop is the floor of this form), 6 us in the epilogue, 2 us until the next tile starts on the unit.
#include <stddef.h>

#include "peqa_device.h"
#include "peqa_kernels.h"

namespace peqa {

namespace {

constexpr int DW_TF = 256;                       // features per workgroup
constexpr int DW_TC = 256;                       // channels per workgroup
constexpr int DW_NST = 4;                        // ring depth
constexpr int DW_A_BYTES = DW_TF * 64;           // 16 KB: 256 feature rows x 32 tokens
constexpr int DW_STAGE = (DW_TF + DW_TC) * 64;   // 32 KB
constexpr int DW_LDS = DW_NST * DW_STAGE;        // 128 KB
constexpr int DW_WM = 4;                         // waves along the features: see dw_kernel

// WM = waves along the features (2: 128 x 128 wave tiles, one wave per SIMD; 4: 64 x 128, two per SIMD)
template <int BITS, int WM>
__device__ __forceinline__ void dw_tile(const DwArgs &a, const int wg, uint8_t *lds)
{
    constexpr int WPB = 2 * BITS;
    constexpr int NRT = 16 / WM;                           // accumulator row tiles per wave
    constexpr int DW_DMA = 16 / WM;                        // DMA instructions per wave per step (32 of 1 KB per stage)
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;              // feature part, channel half
    const int c = lane & 15, q = lane >> 4;

    // workgroup -> tile: the 32 workgroups that run together on one XCD take a patch of 4 feature tiles
    // x 8 channel tiles, so that operand rows are shared through that XCD's L2
    int tile_f, tile_c;
    {
        const int xcd = wg & 7, local = wg >> 3;
        const int g = (local >> 5) * 8 + xcd, r = local & 31;
        const int patches_f = (a.tiles_f + 3) / 4;
        tile_f = (g % patches_f) * 4 + (r & 3);
        tile_c = (g / patches_f) * 8 + (r >> 2);
    }
    if (tile_f >= a.tiles_f || tile_c >= a.tiles_c) return;   // padding of a ragged patch (uniform)

    const int k0 = tile_f * DW_TF, n0 = tile_c * DW_TC;
    const int nsteps = a.Tp >> 5;                          // even: Tp % 64 == 0
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;

    // DMA j of wave w is wave-load d = DW_DMA w + j of the stage: 0..15 = feature rows 16 d .. + 15 of Xt,
    // 16..31 = channel rows 16 (d - 16) .. of dYt.  Lane s lands at row s / 4, chunk position s % 4 and
    // fetches the chunk that the swizzle assigns there.  Rows past the matrix are clamped to its last
    // row: their products are computed and dropped.
    uint32_t voff[DW_DMA];
    const uint8_t *src = reinterpret_cast<const uint8_t *>(wave < WM ? a.Xt : a.dYt);
    const size_t step_bytes = (size_t)(wave < WM ? a.K : a.N) * 64;   // one 32-token step of all rows
    {
        const int row_l = lane >> 2, pos = lane & 3;
        const uint32_t chunk = (uint32_t)(pos ^ a_swizzle(row_l));
        const int first = wave < WM ? k0 : n0, limit = (wave < WM ? a.K : a.N) - 1;
#pragma unroll
        for (int j = 0; j < DW_DMA; ++j) {
            int row = first + 16 * (DW_DMA * (wave % WM) + j) + row_l;
            row = row < limit ? row : limit;
            voff[j] = (uint32_t)row * 64u + chunk * 16u;
        }
    }
    // The queue runs four stages past the last step, so that the DMA count per step is constant.  Of those, the
    // stage numbered `nsteps` carries the packed codes of the tile's 256 x 256 weights for the epilogue: the two runs of
    // 8 step tiles (RUN bytes each: contiguous in the tile-major layout) of its two 128-channel tile rows, copied
    // linearly, KB number d by DMA d = DW_DMA wave + j; the others re-fetch the last step.  Runs past the matrix
    // (second tile row beyond N, step tiles beyond K, the KBs after the two runs at 3 bits) are read from valid
    // memory somewhere else and never looked at.
    constexpr uint32_t CODE_TILE = 64 * WPB * 4, CODE_RUN = 8 * CODE_TILE;   // one 128 x 32 tile; 8 of them (12 or 16 KB)
    const uint8_t *code_src[DW_DMA];
    {
        const size_t total = (size_t)a.N * a.K / 8 * BITS, row_bytes = (size_t)(a.K >> 5) * CODE_TILE;
#pragma unroll
        for (int j = 0; j < DW_DMA; ++j) {
            const uint32_t byte = (uint32_t)(DW_DMA * wave + j) * 1024u;
            uint32_t run = byte / CODE_RUN;
            const uint32_t off = byte - run * CODE_RUN;
            if (run > 1 || (2 * tile_c + (int)run) * 128 >= a.N) run = 0;
            size_t g = (size_t)(2 * tile_c + run) * row_bytes + (size_t)tile_f * CODE_RUN + off;
            g = g + 1024 <= total ? g : total - 1024;
            code_src[j] = reinterpret_cast<const uint8_t *>(a.packed) + g;
        }
    }
    auto issue_one = [&](int j, int it, int stage) {
        const uint32_t dst = lds_base + stage * DW_STAGE + (DW_DMA * wave + j) * 1024;
        if (it == nsteps) {
            dma16((uint32_t)lane * 16u, code_src[j], dst);
        } else {
            const int s = it < nsteps ? it : nsteps - 1;
            dma16(voff[j], src + (size_t)s * step_bytes, dst);
        }
    };
    auto issue = [&](int it, int stage) {
#pragma unroll
        for (int j = 0; j < DW_DMA; ++j) issue_one(j, it, stage);
    };

    f32x4 acc[NRT][8];
#pragma unroll
    for (int i = 0; i < NRT; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int sw = (q ^ a_swizzle(c)) << 4;
    const int a_off = (16 * NRT * wm + c) * 64 + sw;       // + rt * 1024
    const int b_off = DW_A_BYTES + (128 * wn + c) * 64 + sw;   // + ct * 1024
    auto read_a = [&](int stage, int rt) {
        return *reinterpret_cast<const u32x4 *>(lds + stage * DW_STAGE + a_off + rt * 1024);
    };
    auto read_b = [&](int stage, int ct) {
        return *reinterpret_cast<const u32x4 *>(lds + stage * DW_STAGE + b_off + ct * 1024);
    };

    // ---- prologue: four stages queued; the first two complete before the first fragments are read
    issue(0, 0);
    issue(1, 1);
    issue(2, 2);
    issue(3, 3);
    wait_vmcnt<2 * DW_DMA>();
    __syncthreads();
    u32x4 afrag[2][NRT], bfrag[8];
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) afrag[0][rt] = read_a(0, rt);
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) bfrag[ct] = read_b(0, ct);
    // step 0 refills stage 0: every wave must have taken its fragments out of it
    __syncthreads();

    // ---- main loop.  At the start of step `it` its fragments are in registers and stage it + 1 is
    // complete and visible.  The step queues stage it + 4 into its own slot (its fragments left that slot
    // during step it - 1, before the last barrier) while it runs its matrix instructions column tile by
    // column tile, and refills every fragment from stage it + 1 right after its last use.  The closing
    // wait leaves the DMAs of this step and the one before outstanding: stage it + 2 has landed, three
    // steps after it was queued; the barrier makes it visible.
    int cur = 0;
    auto step = [&](int it, auto cur_c) {
        constexpr int CUR = decltype(cur_c)::value, NXT = CUR ^ 1;
        const int nstage = (cur + 1) & (DW_NST - 1);
        static_for<8>([&](auto ct_c) {
            constexpr int ct = ct_c.value;
            static_for<NRT>([&](auto rt_c) { mfma16_acc(acc[rt_c.value][ct], afrag[CUR][rt_c.value], bfrag[ct]); });
            // the DMAs are spread over the step: queued in one burst after the barrier, they hold back the
            // matrix instructions behind them until the memory pipe has taken all of them
            if constexpr (ct % (8 / DW_DMA) == 0) issue_one(ct / (8 / DW_DMA), it + 4, cur);
            bfrag[ct] = read_b(nstage, ct);
            // the next step's first matrix instructions need all its row fragments: those are fetched in
            // the first half of this step, so that only a column fragment is still on its way at the barrier
            if constexpr (ct < 4) {
                static_for<NRT / 4>([&](auto e_c) {
                    constexpr int rt = ct * (NRT / 4) + e_c.value;
                    afrag[NXT][rt] = read_a(nstage, rt);
                });
            }
        });
        wait_vmcnt<2 * DW_DMA>();
        bare_barrier();
        cur = nstage;
    };
    for (int it = 0; it < nsteps; it += 2) {
        step(it, std::integral_constant<int, 0>{});
        step(it + 1, std::integral_constant<int, 1>{});
    }
    wait_vmcnt<0>();
    __syncthreads();
    mfma_result_fence();

    // ---- epilogue: this wave's features are the chunks fb / 64 + h (accumulator rows rt = 4 h .. 4 h + 3);
    // lane (c, q) holds, per accumulator tile (rt, ct), features fb + 16 rt + 4 q + j (j = 0..3) of
    // channel cb + 16 ct + c
    const int fb = k0 + 16 * NRT * wm, cb = n0 + 128 * wn;
    if (cb >= a.N) return;                                 // wave-uniform (N % 128 == 0)
    const int nchunks = a.K >> 6;
    // the tile's codes, in the ring slot of stage `nsteps`: run wn = this wave's 128 channels
    const uint8_t *code_lds = lds + (nsteps & (DW_NST - 1)) * DW_STAGE + wn * CODE_RUN;
    // The lane's four features of an accumulator tile are half a row of one 8 x 8 code block: row r = c % 8 (cb is a
    // multiple of 128), columns 4 hq .. 4 hq + 3 with hq = q % 2 (fb + 16 rt is a multiple of 16).  Where those four
    // codes sit inside the block's words depends on (r, hq) only: worked out once per lane, so that a tile costs a few
    // loads at fixed offsets and shifts by lane constants (taken code by code with run-time row and column, the
    // epilogue took a third of the kernel's time at T = 2048).
    //   4 bits: word r, code of column cc at bits [4 p, 4 p + 4), p = cc / 2 + 4 (cc % 2): after a shift by 8 hq the four
    //           codes are at bits 0, 16, 4, 20.
    //   3 bits: cell u = 4 (r / 2) + cc / 2 holds columns cc = 2 (u % 4), 2 (u % 4) + 1 in its low and high half-word:
    //           the lane has cells u0 = 4 (r / 2) + 2 hq and u0 + 1; cell u < 15 is field u % 5 of word 2 (u / 5) + r % 2,
    //           cell 15 is spread over the top bits of the half-words of words r % 2, 2 + r % 2, 4 + r % 2.
    const int r = c & 7, par = r & 1, hq = q & 1;
    const int u0 = 4 * (r >> 1) + 2 * hq, u1 = u0 + 1;
    const bool spare = u1 == 15;
    // word (within the block) and shift of the lane's two cells; the spare cell is put together in the same form
    // (low code at bit 0, high code at bit 16) from the top bits of the three words
    const int wi0 = 2 * (u0 / 5) + par, sh0 = 3 * (u0 % 5);
    const int wi1 = spare ? par : 2 * (u1 / 5) + par, sh1 = spare ? 0 : 3 * (u1 % 5);
    // one byte of a register to fp32 in one instruction (v_cvt_f32_ubyte0 / 2)
    auto byte0 = [](uint32_t v) { return (float)(v & 0xFFu); };
    auto byte2 = [](uint32_t v) { return (float)((v >> 16) & 0xFFu); };
    auto lane_codes = [&](const uint32_t *blk, float *code) {
        if constexpr (BITS == 4) {
            const uint32_t w = blk[r] >> (8 * hq);
            const uint32_t t0 = w & 0x000F000Fu, t1 = (w >> 4) & 0x000F000Fu;
            code[0] = byte0(t0);
            code[1] = byte2(t0);
            code[2] = byte0(t1);
            code[3] = byte2(t1);
        } else {
            const uint32_t A = blk[par], B = blk[2 + par], C = blk[4 + par];
            const uint32_t S = ((A >> 15) & 0x00010001u) | ((B >> 14) & 0x00020002u) | ((C >> 13) & 0x00040004u);
            const uint32_t t0 = (blk[wi0] >> sh0) & 0x00070007u;
            const uint32_t t1 = ((spare ? S : blk[wi1]) >> sh1) & 0x00070007u;
            code[0] = byte0(t0);
            code[1] = byte2(t0);
            code[2] = byte0(t1);
            code[3] = byte2(t1);
        }
    };
    static_for<NRT / 4>([&](auto h_c) {
        constexpr int h = h_c.value;
        const int fh = fb + 64 * h;
        if (fh >= a.K) return;                             // wave-uniform (K % 64 == 0)
        const int chunk = fh >> 6, grp = fh / a.gsz;
        // zero-points of the lane's eight channels, fetched together and by every lane: inside the q == 0 branch below
        // each would be a load of its own with a full memory latency in front of the store
        float zv[8];
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) {
            const size_t sg = (size_t)(cb + 16 * ct + c) * a.G + grp;
            zv[ct] = (float)a.z0[sg] + (a.dz ? a.dz[sg] : 0.f);
        }
        static_for<8>([&](auto ct_c) {
            constexpr int ct = ct_c.value;
            const int i = cb + 16 * ct + c;
            // blocks of channel block (i / 8) % 16 = 2 ct + c / 8 within the tiles of the run
            const uint32_t *ch_tile = reinterpret_cast<const uint32_t *>(code_lds) + (2 * ct + (c >> 3)) * 4 * WPB;
            float s1 = 0.f, s0 = 0.f;
            static_for<4>([&](auto r_c) {
                constexpr int rt = 4 * h + r_c.value;
                const f32x4 v = read_acc(acc[rt][ct]);
                // the lane's features fb + 16 rt + 4 q + j: step tile (fb - k0 + 16 rt) / 32 of the run, block column
                // 2 (rt % 2) + q / 2
                const uint32_t *blk = ch_tile + (((fb - k0) >> 5) + (rt >> 1)) * 64 * WPB + (2 * (rt & 1) + (q >> 1)) * WPB;
                float code[4];
                lane_codes(blk, code);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    s1 += v[j] * code[j];
                    s0 += v[j];
                }
            });
            s1 += __shfl_xor(s1, 16); s0 += __shfl_xor(s0, 16);
            s1 += __shfl_xor(s1, 32); s0 += __shfl_xor(s0, 32);
            if (q == 0) a.pc[(size_t)i * nchunks + chunk] = s1 - zv[ct] * s0;
        });
    });
}

template <int BITS, int WM>
__global__ __launch_bounds__(128 * WM, 1) void dw_kernel(DwArgs a)
{
    extern __shared__ __align__(16) uint8_t lds[];
    dw_tile<BITS, WM>(a, (int)blockIdx.x, lds);
}

// The token contractions of several layers in one launch: the tiles of job 0 first, then job 1's, ...  One layer's
// tiles alone often fill the machine a fraction over a whole number of times (400 tiles of 256 x 256 on 256 compute
// units for a 5120 x 5120 layer); together only the last round of the launch is partly filled.
template <int BITS, int WM>
__global__ __launch_bounds__(128 * WM, 1) void dw_multi_kernel(DwMultiArgs m)
{
    extern __shared__ __align__(16) uint8_t lds[];
    const int b = (int)blockIdx.x;
    int j = 0, wg0 = 0;
#pragma unroll
    for (int i = 0; i < DW_MAX_JOBS - 1; ++i) {
        const int e = m.wg_end[i];
        if (b >= e) { j = i + 1; wg0 = e; }
    }
    const DwArgs a = kernarg_load<DwArgs>((uint32_t)(j * sizeof(DwArgs)));
    dw_tile<BITS, WM>(a, b - wg0, lds);
}

// transpose_pad_tile (peqa_device.h) for every 64 x 64 tile of src [T, C] (Tp / 64 x C / 64 workgroups).
__global__ __launch_bounds__(256) void transpose_pad_kernel(const uint16_t *__restrict__ src, int T, int C, int Tp,
                                                             uint16_t *__restrict__ dst)
{
    __shared__ uint16_t tile[64][64 + 2];
    transpose_pad_tile(src, T, C, dst, (int)blockIdx.x, (int)blockIdx.y, tile);
}

// d_ds[i, g] = sum of pc[i, chunk] over the gsz / 64 chunks of group g, in order.
__global__ __launch_bounds__(256) void chunk_reduce_kernel(const float *__restrict__ pc, size_t n, int per,
                                                            float *__restrict__ d_ds)
{
    const size_t j = (size_t)blockIdx.x * 256 + threadIdx.x;   // = i * G + g; the chunks of j are contiguous
    if (j >= n) return;
    float s = 0.f;
    for (int e = 0; e < per; ++e) s += pc[j * per + e];
    d_ds[j] = s;
}

// chunk_reduce_kernel for the jobs of a dw_multi launch: blockIdx.y = job.
__global__ __launch_bounds__(256) void chunk_reduce_multi_kernel(DwMultiArgs m)
{
    const DwArgs a = kernarg_load<DwArgs>((uint32_t)(blockIdx.y * sizeof(DwArgs)));
    float *d_ds = m.d_ds[0];
#pragma unroll
    for (int i = 1; i < DW_MAX_JOBS; ++i)
        if ((int)blockIdx.y == i) d_ds = m.d_ds[i];
    const size_t n = (size_t)a.N * a.G;
    const int per = a.gsz >> 6;
    const size_t j = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    float s = 0.f;
    for (int e = 0; e < per; ++e) s += a.pc[j * per + e];
    d_ds[j] = s;
}

constexpr int kMaxDev = 64;
bool g_attr_done[2][kMaxDev];
bool g_attr_done_multi[2][kMaxDev];

}  // namespace

static bool dw_args_ok(const DwArgs &a);

hipError_t launch_transpose_pad(const uint16_t *src, int T, int C, int Tp, uint16_t *dst, hipStream_t stream)
{
    trace_before(KID_TRANSPOSE, stream);
    hipLaunchKernelGGL(transpose_pad_kernel, dim3(Tp / 64, C / 64), dim3(256), 0, stream, src, T, C, Tp, dst);
    trace_after(KID_TRANSPOSE, stream);
    return hipGetLastError();
}

hipError_t launch_dw(int bits, const DwArgs &a, hipStream_t stream)
{
    // what the kernel's indexing assumes
    if (!dw_args_ok(a)) return hipErrorInvalidValue;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDev) return hipErrorInvalidDevice;
    auto kern = bits == 4 ? dw_kernel<4, DW_WM> : dw_kernel<3, DW_WM>;
    bool &done = g_attr_done[bits == 4][dev];
    if (!done) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, DW_LDS);
        if (e != hipSuccess) return e;
        done = true;
    }
    // patches of 4 x 8 tiles, 32 workgroup ids per patch and XCD
    const int patches_f = (a.tiles_f + 3) / 4, patches_c = (a.tiles_c + 7) / 8;
    const int npatch = patches_f * patches_c;
    const unsigned grid = (unsigned)(((npatch + 7) / 8) * 8 * 32);
    trace_before(KID_GEMM_DW, stream);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(128 * DW_WM), DW_LDS, stream, a);
    trace_after(KID_GEMM_DW, stream);
    return hipGetLastError();
}

static bool dw_args_ok(const DwArgs &a)
{
    if (a.K % 64 != 0 || a.N % 128 != 0 || a.Tp % 64 != 0 || a.Tp < 64 || a.gsz % 64 != 0 || a.K % a.gsz != 0) return false;
    return (uint64_t)(a.K > a.N ? a.K : a.N) * 64u < ((uint64_t)1 << 32);   // 32-bit DMA offsets
}

hipError_t launch_dw_multi(int bits, DwMultiArgs &m, hipStream_t stream)
{
    if (m.n_jobs < 1 || m.n_jobs > DW_MAX_JOBS) return hipErrorInvalidValue;
    int total = 0;
    for (int j = 0; j < DW_MAX_JOBS; ++j) {
        if (j < m.n_jobs) {
            const DwArgs &a = m.job[j];
            if (!dw_args_ok(a)) return hipErrorInvalidValue;
            const int patches_f = (a.tiles_f + 3) / 4, patches_c = (a.tiles_c + 7) / 8;
            total += ((patches_f * patches_c + 7) / 8) * 8 * 32;
        } else {
            m.job[j] = m.job[m.n_jobs - 1];
            m.d_ds[j] = m.d_ds[m.n_jobs - 1];
        }
        m.wg_end[j] = total;
    }
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDev) return hipErrorInvalidDevice;
    auto kern = bits == 4 ? dw_multi_kernel<4, DW_WM> : dw_multi_kernel<3, DW_WM>;
    bool &done = g_attr_done_multi[bits == 4][dev];
    if (!done) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, DW_LDS);
        if (e != hipSuccess) return e;
        done = true;
    }
    trace_before(KID_GEMM_DW, stream);
    hipLaunchKernelGGL(kern, dim3(total), dim3(128 * DW_WM), DW_LDS, stream, m);
    trace_after(KID_GEMM_DW, stream);
    return hipGetLastError();
}

hipError_t launch_chunk_reduce_multi(const DwMultiArgs &m, hipStream_t stream)
{
    size_t nmax = 0;
    for (int j = 0; j < m.n_jobs; ++j) {
        const size_t n = (size_t)m.job[j].N * m.job[j].G;
        nmax = n > nmax ? n : nmax;
    }
    trace_before(KID_REDUCE, stream);
    hipLaunchKernelGGL(chunk_reduce_multi_kernel, dim3((unsigned)((nmax + 255) / 256), m.n_jobs), dim3(256), 0, stream, m);
    trace_after(KID_REDUCE, stream);
    return hipGetLastError();
}

hipError_t launch_chunk_reduce(const float *pc, size_t n, int per, float *d_ds, hipStream_t stream)
{
    trace_before(KID_REDUCE, stream);
    hipLaunchKernelGGL(chunk_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, pc, n, per, d_ds);
    trace_after(KID_REDUCE, stream);
    return hipGetLastError();
}

}  // namespace peqa
