// Bandwidth-bound helper kernels around the MFMA contractions: row sums of X, the scaled
// copy of dY, the fixed-order reduction of scale-gradient partials, and the AdamW step.
#include "peqa_device.h"
#include "peqa_kernels.h"

namespace peqa {

namespace {

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// rs[t, h] = sum of X[t, k] over contraction half h (k < ksplit, k >= ksplit), fp32.
// One wave per token row; 16-byte loads.
__device__ __forceinline__ void rowsum_rows(const uint16_t *__restrict__ X, int T, int K, int ksplit, float *__restrict__ rs)
{
    const int lane = threadIdx.x & 63, t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const u32x4 *row = reinterpret_cast<const u32x4 *>(X + (size_t)t * K);
    float s[2] = {0.f, 0.f};
    const int split8 = ksplit >> 3;
    const int n8 = K >> 3;
    // four 16-byte loads of a lane in flight; chunks past the row's end re-read its first chunk and add nothing
    for (int k8 = lane; k8 < n8; k8 += 256) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = row[k8 + 64 * u < n8 ? k8 + 64 * u : 0];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float p = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) p += bf16_lo(v[u][i]) + bf16_hi(v[u][i]);
            const int kk = k8 + 64 * u;
            s[0] += kk < split8 ? p : 0.f;
            s[1] += kk >= split8 && kk < n8 ? p : 0.f;
        }
    }
    s[0] = wave_sum(s[0]);
    s[1] = wave_sum(s[1]);
    if (lane == 0) { rs[2 * t] = s[0]; rs[2 * t + 1] = s[1]; }
}

__global__ __launch_bounds__(256) void rowsum_kernel(const uint16_t *__restrict__ X, int T, int K, int ksplit,
                                                      float *__restrict__ rs)
{
    rowsum_rows(X, T, K, ksplit, rs);
}

// rowsum_kernel's work for several inputs of T rows each: blockIdx.y selects the input.
__global__ __launch_bounds__(256) void rowsum_multi_kernel(RowsumMulti a)
{
    const int y = blockIdx.y;
    const uint16_t *X = a.X[0];
    float *rs = a.rs[0];
    int K = a.K[0];
#pragma unroll
    for (int i = 1; i < ROWSUM_MAX; ++i)
        if (y == i) { X = a.X[i]; rs = a.rs[i]; K = a.K[i]; }
    rowsum_rows(X, a.T, K, K / 2, rs);
}

// rsg[t, g] = sum of X[t, k] over scale group g (gsz features, a multiple of 64), fp32.
// One wave per token row: 8 lanes sum each run of 64 features, the run sums meet in LDS,
// and every group adds its gsz / 64 runs in order.
__global__ __launch_bounds__(256) void rowsum_groups_kernel(const uint16_t *__restrict__ X, int T, int K, int gsz,
                                                             float *__restrict__ rsg)
{
    extern __shared__ float runsum[];                      // [4 waves][K / 64]
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, t = blockIdx.x * 4 + w;
    const int nruns = K >> 6;
    float *mine = runsum + w * nruns;
    if (t < T) {
        const u32x4 *row = reinterpret_cast<const u32x4 *>(X + (size_t)t * K);
        for (int k8 = lane; k8 < (K >> 3); k8 += 64) {    // K % 128 == 0: whole 8-lane segments
            const u32x4 v = row[k8];
            float p = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) p += bf16_lo(v[i]) + bf16_hi(v[i]);
#pragma unroll
            for (int o = 4; o >= 1; o >>= 1) p += __shfl_xor(p, o);
            if ((lane & 7) == 0) mine[k8 >> 3] = p;
        }
    }
    __syncthreads();
    if (t < T) {
        const int per = gsz >> 6, G = K / gsz;
        for (int g = lane; g < G; g += 64) {
            float r = 0.f;
            for (int b = 0; b < per; ++b) r += mine[g * per + b];
            rsg[(size_t)t * G + g] = r;
        }
    }
}

// Entry j = n * G + g of the per-group table from which the grouped contractions take their scales, with
// s = (s0 + ds)[n, g] and z = (z0 + dz)[n, g].
//   a_side = 0:  sb[g][n] = (s, -s (16 + z)): the weights are scaled in the loop (forward, dX)
//   a_side = 1:  sb[g][n / 128] = 1 KB: the 128 scales s of channels 128 (n / 128) .. + 127, then their 128 offsets
//                16 + z as bf16 (exact: integer zero-points only), then 256 bytes never read: what a dX tile that scales
//                its activation fragments fetches per block of channels
__device__ __forceinline__ void group_table_entry(const float *__restrict__ s0, const float *__restrict__ ds,
                                                  const uint8_t *__restrict__ z0, const float *__restrict__ dz, int N,
                                                  int G, int a_side, float *__restrict__ sb, size_t j)
{
    const size_t n = j / G, g = j - n * G;
    const float s = ds ? s0[j] + ds[j] : s0[j];
    const float zoff = kCodeOffset + (float)z0[j] + (dz ? dz[j] : 0.f);
    if (a_side) {
        float *blk = sb + (g * (size_t)(N >> 7) + (n >> 7)) * 256;
        blk[n & 127] = s;
        reinterpret_cast<uint16_t *>(blk + 128)[n & 127] = (uint16_t)float_to_bf16_bits(zoff);
    } else {
        float *o = sb + (g * N + n) * 2;
        o[0] = s;
        o[1] = -s * zoff;
    }
}

__global__ __launch_bounds__(256) void group_table_kernel(const float *__restrict__ s0, const float *__restrict__ ds,
                                                           const uint8_t *__restrict__ z0, const float *__restrict__ dz,
                                                           int N, int G, int a_side, float *__restrict__ sb)
{
    const size_t j = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= (size_t)N * G) return;
    group_table_entry(s0, ds, z0, dz, N, G, a_side, sb, j);
}

// The same table by workgroups of GT_CH channels x all groups, through LDS: memory has a channel's groups next to each
// other and the table a group's channels, so entry by entry every 8-byte write is a transaction of its own (25 us for
// the four tables of a 13B block); here the reads run along the groups and the writes along the channels, 128 bytes
// per group.  `lds`: 2 x GT_CH x G floats.
constexpr int GT_CH = 16;
__device__ __forceinline__ void group_table_tile(const float *__restrict__ s0, const float *__restrict__ ds,
                                                 const uint8_t *__restrict__ z0, const float *__restrict__ dz, int N, int G,
                                                 int a_side, float *__restrict__ sb, int n0, float *lds)
{
    float *s_l = lds, *z_l = lds + GT_CH * G;
    const size_t base = (size_t)n0 * G;
    for (int e = threadIdx.x; e < GT_CH * G; e += 256) {
        const size_t j = base + e;
        s_l[e] = ds ? s0[j] + ds[j] : s0[j];
        z_l[e] = kCodeOffset + (float)z0[j] + (dz ? dz[j] : 0.f);
    }
    __syncthreads();
    const int nl = threadIdx.x % GT_CH, n = n0 + nl;
    for (int g = threadIdx.x / GT_CH; g < G; g += 256 / GT_CH) {
        const float s = s_l[nl * G + g], zoff = z_l[nl * G + g];
        if (a_side) {
            float *blk = sb + ((size_t)g * (size_t)(N >> 7) + (n >> 7)) * 256;
            blk[n & 127] = s;
            reinterpret_cast<uint16_t *>(blk + 128)[n & 127] = (uint16_t)float_to_bf16_bits(zoff);
        } else {
            f32x2 o;
            o[0] = s;
            o[1] = -s * zoff;
            *reinterpret_cast<f32x2 *>(sb + ((size_t)g * N + n) * 2) = o;
        }
    }
}

__global__ __launch_bounds__(256) void group_table_tile_kernel(const float *__restrict__ s0, const float *__restrict__ ds,
                                                                const uint8_t *__restrict__ z0, const float *__restrict__ dz,
                                                                int N, int G, int a_side, float *__restrict__ sb)
{
    extern __shared__ __align__(16) float gt_lds[];
    group_table_tile(s0, ds, z0, dz, N, G, a_side, sb, (int)blockIdx.x * GT_CH, gt_lds);
}

// group_table_tile_kernel for several layers: blockIdx.y = layer.
__global__ __launch_bounds__(256) void group_table_multi_kernel(GroupTableMulti a)
{
    extern __shared__ __align__(16) float gt_lds[];
    const int y = blockIdx.y;
    const float *s0 = a.s0[0], *ds = a.ds[0];
    const uint8_t *z0 = a.z0[0];
    float *sb = a.sb[0];
    int N = a.N[0], G = a.G[0], a_side = a.a_side[0];
#pragma unroll
    for (int i = 1; i < GT_MAX; ++i)
        if (y == i) { s0 = a.s0[i]; ds = a.ds[i]; z0 = a.z0[i]; sb = a.sb[i]; N = a.N[i]; G = a.G[i]; a_side = a.a_side[i]; }
    const int n0 = (int)blockIdx.x * GT_CH;
    if (n0 >= N) return;                                   // uniform per workgroup
    group_table_tile(s0, ds, z0, nullptr, N, G, a_side, sb, n0, gt_lds);
}

// the same entry by entry, for rows of more groups than the tile form's LDS holds
__global__ __launch_bounds__(256) void group_table_multi_entry_kernel(GroupTableMulti a)
{
    const int y = blockIdx.y;
    const float *s0 = a.s0[0], *ds = a.ds[0];
    const uint8_t *z0 = a.z0[0];
    float *sb = a.sb[0];
    int N = a.N[0], G = a.G[0], a_side = a.a_side[0];
#pragma unroll
    for (int i = 1; i < GT_MAX; ++i)
        if (y == i) { s0 = a.s0[i]; ds = a.ds[i]; z0 = a.z0[i]; sb = a.sb[i]; N = a.N[i]; G = a.G[i]; a_side = a.a_side[i]; }
    const size_t j = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= (size_t)N * G) return;
    group_table_entry(s0, ds, z0, nullptr, N, G, a_side, sb, j);
}

// scale_dy_rows (peqa_device.h) for every block of SDY_ROWS token rows.  Workgroups past the last row block do an
// independent job in the same launch: the fixed-order sum of the scale-gradient partials (n_red = 0: none),
// which the backward needs between its two contractions too.
__global__ __launch_bounds__(256) void scale_dy_kernel(const uint16_t *__restrict__ dY, const float *__restrict__ s0,
                                                        const float *__restrict__ ds, const uint8_t *__restrict__ z0,
                                                        const float *__restrict__ dz, int T, int N,
                                                        uint16_t *__restrict__ dYs, float *__restrict__ crow,
                                                        const float *__restrict__ partial, int ntiles, size_t n_red,
                                                        float *__restrict__ red_out)
{
    __shared__ float red[SDY_ROWS * 4];
    const int row_blocks = (T + SDY_ROWS - 1) / SDY_ROWS;
    if ((int)blockIdx.x >= row_blocks) {
        reduce_partials_at(partial, ntiles, n_red, (size_t)((int)blockIdx.x - row_blocks) * 256 + threadIdx.x, red_out);
        return;
    }
    scale_dy_rows(dY, s0, ds, z0, dz, T, N, dYs, crow, (int)blockIdx.x, red);
}

// Scale gradient from the product P[t,i] = sum_k X[t,k] (Q[i,k] - z0[i]) that the forward kept:
// partial[slice, i] = sum of dY[t,i] P[t,i] over the KEPT_ROWS token rows of the slice.  A workgroup
// takes 256 channels (4 per lane) of one slice; wave w adds rows w, w+4, ... in order and the four
// wave sums meet in LDS in a fixed order.
__global__ __launch_bounds__(256) void dds_kept_kernel(const uint16_t *__restrict__ dY, const float *__restrict__ P,
                                                        int T, int N, float *__restrict__ partial)
{
    __shared__ f32x4 part[4][64];
    const int q = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int col = blockIdx.y * 256 + 4 * q;
    const int tbeg = blockIdx.x * KEPT_ROWS;
    const int nrows = min(KEPT_ROWS, T - tbeg);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    if (col < N) {
        const size_t base = (size_t)tbeg * N + col;
#pragma unroll 4
        for (int r = w; r < nrows; r += 4) {
            const u32x2 d = *reinterpret_cast<const u32x2 *>(dY + base + (size_t)r * N);
            const f32x4 p = *reinterpret_cast<const f32x4 *>(P + base + (size_t)r * N);
            acc[0] += bf16_lo(d[0]) * p[0];
            acc[1] += bf16_hi(d[0]) * p[1];
            acc[2] += bf16_lo(d[1]) * p[2];
            acc[3] += bf16_hi(d[1]) * p[3];
        }
    }
    part[w][q] = acc;
    __syncthreads();
    if (w == 0 && col < N) {
        const f32x4 s = ((part[0][q] + part[1][q]) + part[2][q]) + part[3][q];
        *reinterpret_cast<f32x4 *>(partial + (size_t)blockIdx.x * N + col) = s;
    }
}

// Zero-point gradient, first stage (Appendix K trains zero-points too; z enters Eq. 2 only through -s z, so
// d_dz[i,g] = -s[i,g] * sum_t dY[t,i] R[t,g] with R[t,g] the sum of X[t,k] over scale group g):
// partial[slice, i, g] = sum over the slice's KEPT_ROWS token rows of dY[t,i] * R[t,g].
// A workgroup takes 256 channels (4 per lane) of one slice and walks the groups 8 at a time; wave w
// adds rows w, w+4, ... in order; the four wave sums meet in LDS in a fixed order.
__global__ __launch_bounds__(256) void dz_partial_kernel(const uint16_t *__restrict__ dY, const float *__restrict__ rsg,
                                                          int T, int N, int G, float *__restrict__ partial)
{
    __shared__ float part[4][32][64];                        // [wave][channel-in-lane * 8 + group][lane]
    const int q = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = blockIdx.y * 256 + 4 * q;
    const int tbeg = blockIdx.x * KEPT_ROWS;
    const int nrows = min(KEPT_ROWS, T - tbeg);
    const bool on = col < N;
    for (int gc = 0; gc < G; gc += 8) {
        float acc[4][8];
#pragma unroll
        for (int cc = 0; cc < 4; ++cc)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[cc][j] = 0.f;
        if (on) {
            for (int r = w; r < nrows; r += 4) {
                const size_t t = (size_t)(tbeg + r);
                const u32x2 d = *reinterpret_cast<const u32x2 *>(dY + t * N + col);
                const float dv[4] = {bf16_lo(d[0]), bf16_hi(d[0]), bf16_lo(d[1]), bf16_hi(d[1])};
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float R = rsg[t * G + min(gc + j, G - 1)];   // groups past G are dropped at the store
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc) acc[cc][j] += dv[cc] * R;
                }
            }
        }
        __syncthreads();                                     // the previous chunk's sums have been read
#pragma unroll
        for (int cc = 0; cc < 4; ++cc)
#pragma unroll
            for (int j = 0; j < 8; ++j) part[w][cc * 8 + j][q] = acc[cc][j];
        __syncthreads();
        if (w == 0 && on) {
#pragma unroll
            for (int cc = 0; cc < 4; ++cc)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int e = cc * 8 + j;
                    const float s = ((part[0][e][q] + part[1][e][q]) + part[2][e][q]) + part[3][e][q];
                    if (gc + j < G) partial[((size_t)blockIdx.x * N + col + cc) * G + gc + j] = s;
                }
        }
    }
}

// d_dz[j] = -(s0 + ds)[j] * (partial[0][j] + partial[1][j] + ...) in that order.
__global__ __launch_bounds__(256) void dz_finish_kernel(const float *__restrict__ partial, int slices, size_t n,
                                                         const float *__restrict__ s0, const float *__restrict__ ds,
                                                         float *__restrict__ d_dz)
{
    const size_t j = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    float s = 0.f;
    for (int tt = 0; tt < slices; ++tt) s += partial[(size_t)tt * n + j];
    const float sc = ds ? s0[j] + ds[j] : s0[j];
    d_dz[j] = -sc * s;
}

__global__ __launch_bounds__(256) void reduce_partials_kernel(const float *__restrict__ partial, int ntiles, size_t n,
                                                               float *__restrict__ out)
{
    reduce_partials_at(partial, ntiles, n, (size_t)blockIdx.x * 256 + threadIdx.x, out);
}

__global__ __launch_bounds__(256) void adamw_kernel(size_t n, float *__restrict__ ds, const float *__restrict__ g,
                                                     float *__restrict__ m, float *__restrict__ v,
                                                     const float *__restrict__ s0, float lr, float b1, float b2,
                                                     float eps, float wd, float inv_c1, float inv_c2)
{
    const size_t j = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    const float gj = g[j];
    const float mj = b1 * m[j] + (1.f - b1) * gj;
    const float vj = b2 * v[j] + (1.f - b2) * gj * gj;
    m[j] = mj;
    v[j] = vj;
    const float d = ds[j];
    ds[j] = d - lr * ((mj * inv_c1) / (sqrtf(vj * inv_c2) + eps) + wd * (s0[j] + d));
}

// The same update over several parameter vectors laid end to end in one index space.
__global__ __launch_bounds__(256) void adamw_multi_kernel(AdamwMulti a, float lr, float b1, float b2, float eps,
                                                           float wd, float inv_c1, float inv_c2)
{
    const unsigned long long idx = (unsigned long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= a.end[ADAMW_MAX_TENSORS - 1]) return;
    int t = 0;
#pragma unroll
    for (int i = 0; i < ADAMW_MAX_TENSORS - 1; ++i) t += idx >= a.end[i];
    // selects instead of indexing: the argument block stays in scalar registers
    float *ds = a.ds[0]; const float *g = a.g[0]; float *m = a.m[0]; float *v = a.v[0]; const float *s0 = a.s0[0];
    unsigned long long beg = 0;
#pragma unroll
    for (int i = 1; i < ADAMW_MAX_TENSORS; ++i)
        if (t == i) { ds = a.ds[i]; g = a.g[i]; m = a.m[i]; v = a.v[i]; s0 = a.s0[i]; beg = a.end[i - 1]; }
    const size_t j = (size_t)(idx - beg);
    const float gj = g[j];
    const float mj = b1 * m[j] + (1.f - b1) * gj;
    const float vj = b2 * v[j] + (1.f - b2) * gj * gj;
    m[j] = mj;
    v[j] = vj;
    const float d = ds[j];
    ds[j] = d - lr * ((mj * inv_c1) / (sqrtf(vj * inv_c2) + eps) + wd * (s0[j] + d));
}

}  // namespace

hipError_t launch_adamw_multi(const AdamwMulti &a, float lr, float b1, float b2, float eps, float wd, float inv_c1,
                              float inv_c2, hipStream_t stream)
{
    const unsigned long long total = a.end[ADAMW_MAX_TENSORS - 1];
    trace_before(KID_ADAMW, stream);
    hipLaunchKernelGGL(adamw_multi_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, a, lr, b1, b2, eps,
                       wd, inv_c1, inv_c2);
    trace_after(KID_ADAMW, stream);
    return hipGetLastError();
}

hipError_t launch_rowsum(const uint16_t *X, int T, int K, int ksplit, float *rs, hipStream_t stream)
{
    trace_before(KID_ROWSUM, stream);
    hipLaunchKernelGGL(rowsum_kernel, dim3((T + 3) / 4), dim3(256), 0, stream, X, T, K, ksplit, rs);
    trace_after(KID_ROWSUM, stream);
    return hipGetLastError();
}

hipError_t launch_rowsum_multi(const RowsumMulti &a, hipStream_t stream)
{
    trace_before(KID_ROWSUM, stream);
    hipLaunchKernelGGL(rowsum_multi_kernel, dim3((a.T + 3) / 4, a.n), dim3(256), 0, stream, a);
    trace_after(KID_ROWSUM, stream);
    return hipGetLastError();
}

hipError_t launch_rowsum_groups(const uint16_t *X, int T, int K, int gsz, float *rsg, hipStream_t stream)
{
    trace_before(KID_ROWSUM, stream);
    hipLaunchKernelGGL(rowsum_groups_kernel, dim3((T + 3) / 4), dim3(256), (size_t)4 * (K >> 6) * sizeof(float), stream,
                       X, T, K, gsz, rsg);
    trace_after(KID_ROWSUM, stream);
    return hipGetLastError();
}

// most groups per channel the tile form takes (48 KB of LDS)
constexpr int GT_TILE_MAX_G = 48 * 1024 / (2 * GT_CH * (int)sizeof(float));

hipError_t launch_group_table(const float *s0, const float *ds, const uint8_t *z0, const float *dz, int N, int G,
                              bool a_side, float *sb, hipStream_t stream)
{
    trace_before(KID_GROUP_TABLE, stream);
    if (G <= GT_TILE_MAX_G) {
        hipLaunchKernelGGL(group_table_tile_kernel, dim3(N / GT_CH), dim3(256), 2 * GT_CH * G * sizeof(float), stream, s0, ds, z0,
                           dz, N, G, a_side ? 1 : 0, sb);
    } else {
        const size_t n = (size_t)N * G;
        hipLaunchKernelGGL(group_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, s0, ds, z0, dz, N, G,
                           a_side ? 1 : 0, sb);
    }
    trace_after(KID_GROUP_TABLE, stream);
    return hipGetLastError();
}

hipError_t launch_group_table_multi(const GroupTableMulti &a, hipStream_t stream)
{
    size_t nmax = 0;
    int Nmax = 0, Gmax = 0;
    for (int i = 0; i < a.n; ++i) {
        const size_t n = (size_t)a.N[i] * a.G[i];
        nmax = n > nmax ? n : nmax;
        Nmax = a.N[i] > Nmax ? a.N[i] : Nmax;
        Gmax = a.G[i] > Gmax ? a.G[i] : Gmax;
    }
    trace_before(KID_GROUP_TABLE, stream);
    if (Gmax <= GT_TILE_MAX_G)
        hipLaunchKernelGGL(group_table_multi_kernel, dim3(Nmax / GT_CH, a.n), dim3(256), 2 * GT_CH * Gmax * sizeof(float), stream, a);
    else
        hipLaunchKernelGGL(group_table_multi_entry_kernel, dim3((unsigned)((nmax + 255) / 256), a.n), dim3(256), 0, stream, a);
    trace_after(KID_GROUP_TABLE, stream);
    return hipGetLastError();
}

hipError_t launch_scale_dy(const uint16_t *dY, const float *s0, const float *ds, const uint8_t *z0, const float *dz,
                           int T, int N, uint16_t *dYs, float *crow, const float *partial, int ntiles, size_t n_red,
                           float *red_out, hipStream_t stream)
{
    trace_before(KID_SCALE_DY, stream);
    const unsigned blocks = (unsigned)((T + SDY_ROWS - 1) / SDY_ROWS) + (unsigned)((n_red + 255) / 256);
    hipLaunchKernelGGL(scale_dy_kernel, dim3(blocks), dim3(256), 0, stream, dY, s0, ds, z0, dz, T, N, dYs, crow, partial,
                       ntiles, n_red, red_out);
    trace_after(KID_SCALE_DY, stream);
    return hipGetLastError();
}

hipError_t launch_dds_kept(const uint16_t *dY, const float *P, int T, int N, float *partial, hipStream_t stream)
{
    trace_before(KID_DDS_KEPT, stream);
    hipLaunchKernelGGL(dds_kept_kernel, dim3((T + KEPT_ROWS - 1) / KEPT_ROWS, (N + 255) / 256), dim3(256), 0, stream,
                       dY, P, T, N, partial);
    trace_after(KID_DDS_KEPT, stream);
    return hipGetLastError();
}

hipError_t launch_dz_partial(const uint16_t *dY, const float *rsg, int T, int N, int G, float *partial,
                             hipStream_t stream)
{
    trace_before(KID_DZ_PARTIAL, stream);
    hipLaunchKernelGGL(dz_partial_kernel, dim3((T + KEPT_ROWS - 1) / KEPT_ROWS, (N + 255) / 256), dim3(256), 0, stream,
                       dY, rsg, T, N, G, partial);
    trace_after(KID_DZ_PARTIAL, stream);
    return hipGetLastError();
}

hipError_t launch_dz_finish(const float *partial, int slices, size_t n, const float *s0, const float *ds, float *d_dz,
                            hipStream_t stream)
{
    trace_before(KID_DZ_FINISH, stream);
    hipLaunchKernelGGL(dz_finish_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, partial, slices, n,
                       s0, ds, d_dz);
    trace_after(KID_DZ_FINISH, stream);
    return hipGetLastError();
}

hipError_t launch_reduce_partials(const float *partial, int ntiles, size_t n, float *out, hipStream_t stream)
{
    trace_before(KID_REDUCE, stream);
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, partial,
                       ntiles, n, out);
    trace_after(KID_REDUCE, stream);
    return hipGetLastError();
}

hipError_t launch_adamw(size_t n, float *ds, const float *g, float *m, float *v, const float *s0, float lr, float b1,
                        float b2, float eps, float wd, float inv_c1, float inv_c2, hipStream_t stream)
{
    trace_before(KID_ADAMW, stream);
    hipLaunchKernelGGL(adamw_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, n, ds, g, m, v, s0, lr,
                       b1, b2, eps, wd, inv_c1, inv_c2);
    trace_after(KID_ADAMW, stream);
    return hipGetLastError();
}

}  // namespace peqa
