// Internal launch interface between the C-ABI layer (peqa_api.hip) and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace peqa {

enum { MODE_Y = 0, MODE_DDS = 1, MODE_DX = 2 };

// Test and comparison switches, set through peqa_set_option (peqa_api.hip); the defaults select by launch size.
struct Options {
    int gemm_waves = 0;     // 0 = by launch size, 4 or 8 = that form of the tiled contraction
    int bwd_pair = -1;      // -1 = pair the two contractions of a per-channel backward unless gemm_waves is 8; 0, 1 = never, always
    int grouped_dds = 0;    // 0 = group-wise scale gradient by the contraction over tokens, 1 = over features (older route)
};
Options &options();

// Arguments of the tiled MFMA contraction (peqa_gemm.hip).
struct GemmArgs {
    const uint32_t *packed;   // packed codes of the whole layer
    const uint16_t *A;        // activation operand [T, KC] bf16: X (MODE_Y, MODE_DDS) or scaled dY (MODE_DX)
    int T;                    // tokens
    int KC;                   // contraction length: K (MODE_Y/DDS) or N (MODE_DX)
    int C;                    // output columns:     N (MODE_Y/DDS) or K (MODE_DX)
    int K;                    // input features of the layer (fixes the block stride of `packed`)
    int tiles_c, tiles_t;     // ceil(C/256), ceil(T/128)
    int patch_t;              // token tiles per L2 patch (1, 2 or 4; set by launch_gemm)
    const float *s0;          // [N]            (MODE_Y)
    const float *ds;          // [N] or NULL    (MODE_Y)
    const uint8_t *z0;        // [N]            (MODE_Y, MODE_DDS)
    const float *dz;          // [N] or NULL: trained zero-point offset, z = z0 + dz (MODE_Y, MODE_DDS; [N, G] if grouped)
    const float *rs;          // [T, 2] sums of X[t, :] over each contraction half (MODE_Y, MODE_DDS)
    const float *crow;        // [T] sum_i A[t,i] (16 + z_i)                      (MODE_DX)
    const uint16_t *dY;       // [T, N] bf16    (MODE_DDS)
    float *partial;           // [tiles_t, N]   (MODE_DDS) per-token-tile column sums
    // MODE_DX, group-wise, four-wave form only: tp_blocks > 0 adds that many workgroups at the end of the grid, which
    // write the step-major transposed copies of X [T, K] and dY [T, N] (transpose_pad_tile) that the token contraction
    // of the same backward reads afterwards: Tp / 64 x K / 64 tiles of X first, then Tp / 64 x N / 64 of dY
    int tp_blocks, tp_Tp;
    const uint16_t *tp_X;
    uint16_t *tp_Xt, *tp_dYt;
    uint16_t *out;            // [T, C] bf16    (MODE_Y: Y, MODE_DX: dX)
    float *P;                 // [T, N] fp32 or NULL (MODE_Y, per-channel): sum_k X[t,k] (Q[i,k] - z0[i]), kept
    // group-wise layers (gsz > 0; a multiple of 64):
    int N;                    // output channels of the layer
    int gsz, G;               // group size and groups per channel
    const float *sb;          // [G, N, 2] (s0 + ds, -(s0 + ds)(16 + z0))  (MODE_Y, MODE_DX)
    int a_side;               // MODE_DX, four-wave form, gsz % 128 == 0: the scales go on the activation fragments
                              // and sb is the table launch_group_table makes with a_side
                              // rs is then [T, G]: sums of X over every scale group (MODE_DDS),
                              // partial is [tiles_t, N, G] and z0 is [N, G]
};

hipError_t launch_gemm(int bits, int mode, const GemmArgs &a, hipStream_t stream);
// whether a per-channel launch of that many 128 x 256 tiles takes the four-wave form (two workgroups per compute unit);
// for a huge count: whether the four-wave form is allowed at all (the option gemm_waves = 8 forbids it)
bool gemm_four_waves(int tiles);
// Per-channel layers: the MODE_DDS and the MODE_DX contraction of one backward (arguments as for launch_gemm) as one
// launch of four-wave workgroups (measured faster than two launches at every T).  The dX arguments' input (the scaled dY) must be complete before the launch.
hipError_t launch_gemm_bwd_pair(int bits, const GemmArgs &a_dds, const GemmArgs &a_dx, hipStream_t stream);

// Several contractions in ONE launch of four-wave workgroups (gemm_multi_kernel): the tiles of job 0 first, then
// job 1's, ... (the caller orders them by contraction length, longest first, so that the last, partly filled round
// of the launch is made of short tiles).  Per-channel layers only.  Workgroups numbered [aux_begin, aux_begin +
// aux_wgs) do bandwidth-bound side work of the same backward instead of a tile: every one of them walks a share
// of the row blocks of the scale_dy jobs, of the 256-element chunks of the reduce jobs, or of the 64 x 64 tiles of
// the transpose jobs (the operands of the token contraction of group-wise layers).  They sit in the middle
// of the grid, where they start while most compute units still run tiles, so that their memory traffic hides
// behind matrix work.  All job sizes, aux_begin and aux_wgs are multiples of 8 (workgroup id % 8 = XCD throughout).
constexpr int MULTI_MAX_JOBS = 8;
struct MultiJob {
    GemmArgs a;
    int mode;                 // MODE_Y, MODE_DDS or MODE_DX
    int wg_end;               // tile workgroups of this job and all before it (unused entries: the total)
};
constexpr int SDY_ROWS_HOST = 4;      // token rows per row block of scale_dy_rows (checked against the device constant)
struct ScaleDyJob {           // dYs = bf16(dY (s0 + ds)), crow[t] = sum_i dYs[t,i] (16 + z0[i])   (scale_dy_rows)
    const uint16_t *dY;
    const float *s0, *ds;
    const uint8_t *z0;
    uint16_t *dYs;
    float *crow;
    int T, N;
    int blk_end;              // row blocks (of SDY_ROWS rows) of this job and all before it
};
struct ReduceJob {            // out[j] = sum over ntiles of partial[tile][j], fixed order
    const float *partial;
    float *out;
    int ntiles, n;
    int chunk_end;            // 256-element chunks of this job and all before it
};
struct TransposeJob {         // dst[t / 32][c][t % 32] = src[t, c], zero-padded to Tp tokens      (transpose_pad_tile)
    const uint16_t *src;
    uint16_t *dst;
    int T, C, Tp;
    int tile_end;             // 64 x 64 tiles of this job and all before it
};
struct MultiArgs {
    MultiJob job[MULTI_MAX_JOBS];          // must stay the first member: indexed in the argument block
    ScaleDyJob sdy[MULTI_MAX_JOBS];
    ReduceJob red[MULTI_MAX_JOBS];
    TransposeJob tp[2 * MULTI_MAX_JOBS];
    int n_jobs, n_sdy, n_red, n_tp;
    int aux_begin, aux_wgs;
};
// Per-channel jobs (any mode), or, with `grouped`, group-wise MODE_Y / MODE_DX jobs (their tables in a.sb).
static_assert(sizeof(MultiArgs) <= 4096, "kernel argument block");
hipError_t launch_gemm_multi(int bits, bool grouped, MultiArgs &m, hipStream_t stream);
// workgroups a contraction's tiles take in such a launch (a multiple of 8: whole XCD patches)
int gemm_multi_wgs(int tiles_t, int tiles_c);

// Arguments of the token contraction dW = dY^T X with the codes applied in its epilogue (peqa_dw.hip):
// the scale gradient of group-wise layers.
struct DwArgs {
    const uint16_t *Xt;       // [Tp / 32, K, 32] bf16: X transposed in 32-token steps, tokens padded with zeros to Tp
    const uint16_t *dYt;      // [Tp / 32, N, 32] bf16
    const uint32_t *packed;   // packed codes of the layer
    const uint8_t *z0;        // [N, G]
    const float *dz;          // [N, G] or NULL
    float *pc;                // [N, K / 64] out: sum over each 64-feature chunk of dW[i,k] (Q[i,k] - z[i,g(k)])
    int N, K, Tp;             // Tp % 64 == 0
    int gsz, G;               // group size (multiple of 64) and groups per channel
    int tiles_f, tiles_c;     // ceil(K / 256), ceil(N / 256)
};
hipError_t launch_transpose_pad(const uint16_t *src, int T, int C, int Tp, uint16_t *dst, hipStream_t stream);
hipError_t launch_dw(int bits, const DwArgs &a, hipStream_t stream);
hipError_t launch_chunk_reduce(const float *pc, size_t n, int per, float *d_ds, hipStream_t stream);
// The token contractions of up to DW_MAX_JOBS layers in one launch, and the sums of their chunks in another.
constexpr int DW_MAX_JOBS = 8;
struct DwMultiArgs {
    DwArgs job[DW_MAX_JOBS];               // must stay the first member: indexed in the argument block
    int wg_end[DW_MAX_JOBS];               // workgroups of job j and all before it (unused entries: the total)
    float *d_ds[DW_MAX_JOBS];              // [N, G] out of the chunk sums
    int n_jobs;
};
hipError_t launch_dw_multi(int bits, DwMultiArgs &m, hipStream_t stream);
hipError_t launch_chunk_reduce_multi(const DwMultiArgs &m, hipStream_t stream);
// The (s, b) tables of up to GT_MAX layers in one launch.
constexpr int GT_MAX = 8;
struct GroupTableMulti {
    const float *s0[GT_MAX], *ds[GT_MAX];
    const uint8_t *z0[GT_MAX];
    float *sb[GT_MAX];
    int N[GT_MAX], G[GT_MAX], a_side[GT_MAX];
    int n;
};
hipError_t launch_group_table_multi(const GroupTableMulti &a, hipStream_t stream);

// Arguments of the T <= 16 forward (peqa_gemv.hip): up to GEMV_MAX_LAYERS layers in one launch, laid side by
// side along the workgroup index.  Every layer has its own shape, input and slicing, so that the linears of a
// whole decoder block (different K, different X) can share one launch; the bit width is the launch's.
constexpr int GEMV_MAX_LAYERS = 8;
struct GemvLayer {
    const uint32_t *packed;
    const float *s0, *ds;     // [N, G]; ds may be NULL
    const uint8_t *z0;        // [N, G]
    const float *dz;          // [N, G] or NULL: trained zero-point offset
    const uint16_t *X;        // [T, K] bf16
    uint16_t *Y;              // [T, N] bf16
    float *partial;           // [S, T, N] fp32 slice partials of this layer (S > 1)
    int N, K, G;
    int chunk;                // features per scale group (K for per-channel layers)
    int S;                    // feature slices: a channel tile is S workgroups
    int wg_end;               // workgroups of this layer and all before it (unused entries: the total)
};
struct GemvArgs {
    GemvLayer layer[GEMV_MAX_LAYERS];   // must stay the first member: the kernels index it in the argument block
    int n_layers;
    int T;
    int second_from;                    // workgroups from this index on are taken to be the second on their compute
                                        // unit (set by launch_gemv: the number of compute units)
};
// zbyte: no layer of the launch has a trained zero-point offset, so zero-points stay bytes in LDS and a slice may
// span more scale groups
int gemv_slices(int Ntot, int K, int T, int chunk, bool zbyte);
// Slices per layer for a launch of several layers of different shapes: every workgroup gets about the same
// number of packed bytes, and all of them are resident at once.  Fills S[0..n).
void gemv_plan(int n, const int *N, const int *K, const int *chunk, int bits, int T, bool zbyte, int *S);
// whether a per-channel launch of that many channel tiles with a single slice takes the 12-wave workgroups
bool gemv_whole(int tiles, bool per_channel, int S);
hipError_t launch_gemv(int bits, const GemvArgs &a, hipStream_t stream);

// peqa_small.hip
hipError_t launch_rowsum(const uint16_t *X, int T, int K, int ksplit, float *rs, hipStream_t stream);
// the same for up to ROWSUM_MAX inputs of T rows each in one launch
constexpr int ROWSUM_MAX = 8;
struct RowsumMulti {
    const uint16_t *X[ROWSUM_MAX];
    float *rs[ROWSUM_MAX];
    int K[ROWSUM_MAX];
    int n, T;
};
hipError_t launch_rowsum_multi(const RowsumMulti &a, hipStream_t stream);
// dYs = bf16(dY (s0 + ds)) and crow; with n_red > 0 the same launch also sums `ntiles` partial vectors of n_red
// floats into red_out (launch_reduce_partials' job), an independent piece of work of the same backward
hipError_t launch_scale_dy(const uint16_t *dY, const float *s0, const float *ds, const uint8_t *z0, const float *dz,
                           int T, int N, uint16_t *dYs, float *crow, const float *partial, int ntiles, size_t n_red,
                           float *red_out, hipStream_t stream);
hipError_t launch_rowsum_groups(const uint16_t *X, int T, int K, int gsz, float *rsg, hipStream_t stream);
// sb [G, N, 2] = (s, -s (16 + z)); with a_side [G, N / 128] blocks of 1 KB: the 128 scales s of a block of channels,
// then their offsets 16 + z as bf16 (same size in all: 8 N G bytes)
hipError_t launch_group_table(const float *s0, const float *ds, const uint8_t *z0, const float *dz, int N, int G,
                              bool a_side, float *sb, hipStream_t stream);
// zero-point gradient: partial [ceil(T / KEPT_ROWS), N, G] from dY and the group sums rsg [T, G] of X, then
// d_dz[j] = -(s0 + ds)[j] * (sum of the partials)
hipError_t launch_dz_partial(const uint16_t *dY, const float *rsg, int T, int N, int G, float *partial,
                             hipStream_t stream);
hipError_t launch_dz_finish(const float *partial, int slices, size_t n, const float *s0, const float *ds, float *d_dz,
                            hipStream_t stream);
constexpr int KEPT_ROWS = 64;   // token rows per partial of launch_dds_kept
hipError_t launch_dds_kept(const uint16_t *dY, const float *P, int T, int N, float *partial, hipStream_t stream);
hipError_t launch_reduce_partials(const float *partial, int ntiles, size_t n, float *out, hipStream_t stream);
hipError_t launch_adamw(size_t n, float *ds, const float *g, float *m, float *v, const float *s0,
                        float lr, float b1, float b2, float eps, float wd, float inv_c1, float inv_c2,
                        hipStream_t stream);

// AdamW on several parameter vectors in one launch: tensor j holds elements [end[j-1], end[j]) of the
// launch's index space
constexpr int ADAMW_MAX_TENSORS = 16;
struct AdamwMulti {
    float *ds[ADAMW_MAX_TENSORS];
    const float *g[ADAMW_MAX_TENSORS];
    float *m[ADAMW_MAX_TENSORS];
    float *v[ADAMW_MAX_TENSORS];
    const float *s0[ADAMW_MAX_TENSORS];
    unsigned long long end[ADAMW_MAX_TENSORS];   // running totals; unused entries repeat the last
    int n_tensors;
};
hipError_t launch_adamw_multi(const AdamwMulti &a, float lr, float b1, float b2, float eps, float wd, float inv_c1,
                              float inv_c2, hipStream_t stream);

// peqa_quantize.hip
hipError_t launch_quantize(const float *W0, int N, int K, int bits, int group, uint32_t *packed,
                           float *s0, uint8_t *z0, hipStream_t stream);

// error-minimising variant (clipped-range grid); only where the rows fit in registers and LDS
bool quantize_resident_fits(int K, int G, bool search);
hipError_t launch_quantize_search(const float *W0, int N, int K, int bits, int group, int n_ratios, float step,
                                  uint32_t *packed, float *s0, uint8_t *z0, hipStream_t stream);

// Tracing hook: every launch goes through these so that peqa_trace_* can time it.
void trace_before(int kernel_id, hipStream_t stream);
void trace_after(int kernel_id, hipStream_t stream);

enum {
    KID_QUANTIZE = 0, KID_ROWSUM, KID_GEMM_Y, KID_GEMM_DDS, KID_GEMM_DX, KID_SCALE_DY,
    KID_REDUCE, KID_ADAMW, KID_GEMV, KID_GEMV_FINISH, KID_GROUP_TABLE, KID_DDS_KEPT, KID_DZ_PARTIAL, KID_DZ_FINISH, KID_TRANSPOSE, KID_GEMM_DW, KID_GEMM_BWD, KID_GEMM_MULTI_Y, KID_GEMM_MULTI_DDS, KID_GEMM_MULTI_DX, KID_COUNT
};

}  // namespace peqa
