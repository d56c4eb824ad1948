// Eq. 1 of the paper: round-to-nearest asymmetric quantization with a min-max range,
// fused with the dense packing of the codes into 8x8 blocks (layout: peqa_bit_location()).
//
// One workgroup quantizes 8 output channels (one row of blocks).  Pass 1 reduces min/max
// per (channel, group) and derives s0, z0; pass 2 re-reads the rows (from L2), rounds,
// and assembles whole packed words in LDS so that they leave in runs of 4 blocks (a tile row).
// HBM-bound: 4 N K bytes in, N K b / 8 bytes out.
//
// Every fp32 step below is a single IEEE operation (correctly rounded divide, no
// reciprocal, no fused multiply-add), because the codes must match the definition bit
// for bit.
#include "peqa_device.h"
#include "peqa_kernels.h"

namespace peqa {

namespace {

constexpr int CHUNK = 256;    // features per pass-2 step = 32 blocks

template <int BITS>
__global__ __launch_bounds__(256) void quantize_kernel(const float *__restrict__ W0, int K, int gs, int G,
                                                        uint32_t *__restrict__ packed, float *__restrict__ s0,
                                                        uint8_t *__restrict__ z0)
{
    extern __shared__ __align__(16) uint8_t smem[];
    float *s_s = reinterpret_cast<float *>(smem);                       // [8][G]
    int *s_z = reinterpret_cast<int *>(smem + (size_t)8 * G * 4);       // [8][G]
    uint32_t *s_out = reinterpret_cast<uint32_t *>(smem + (size_t)16 * G * 4);   // 4-bit: 256 words; 3-bit: 512 words of codes

    constexpr int qmax = (1 << BITS) - 1;
    constexpr int WPB = 2 * BITS;
    const int tid = threadIdx.x, r = tid >> 5, j = tid & 31;
    const int ib = blockIdx.x;
    const float *row = W0 + (size_t)(ib * 8 + r) * K;

    // ---- pass 1: range -> (s0, z0) per group
    const int L = gs >= 128 ? 32 : gs / 4;       // lanes per group team (gs = 64 -> 16)
    const int teams = 32 / L, team = j / L, jl = j % L;
    for (int g = team; g < G; g += teams) {
        const f32x4 *p = reinterpret_cast<const f32x4 *>(row + (size_t)g * gs);
        float xmin = 0.f, xmax = 0.f;
        for (int k4 = jl; k4 < gs / 4; k4 += L) {
            const f32x4 v = p[k4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (v[i] < xmin) xmin = v[i];
                if (v[i] > xmax) xmax = v[i];
            }
        }
        for (int o = L >> 1; o >= 1; o >>= 1) {
            const float a = __shfl_xor(xmin, o), b = __shfl_xor(xmax, o);
            if (a < xmin) xmin = a;
            if (b > xmax) xmax = b;
        }
        if (jl == 0) {
            const float range = __fsub_rn(xmax, xmin);
            float s = __fdiv_rn(range, (float)qmax);
            int z;
            if (!(s > 0.f)) {
                s = 1.f;
                z = 0;
            } else {
                z = (int)rintf(__fdiv_rn(-xmin, s));
                z = z < 0 ? 0 : (z > qmax ? qmax : z);
            }
            s_s[r * G + g] = s;
            s_z[r * G + g] = z;
            s0[(size_t)(ib * 8 + r) * G + g] = s;
            z0[(size_t)(ib * 8 + r) * G + g] = (uint8_t)z;
        }
    }
    __syncthreads();

    // ---- pass 2: codes and packing, 32 blocks per step
    // block kb of this row of blocks: tile (ib / 16, kb / 4), block (ib % 16) * 4 + kb % 4 of the tile
    const size_t out_row = (size_t)(ib / 16) * (K / 32) * 64 + (size_t)(ib % 16) * 4;
    for (int k0 = 0; k0 < K; k0 += CHUNK) {
        const int nb = (K - k0) / 8 < 32 ? (K - k0) / 8 : 32;
        if (j < nb) {
            const int k = k0 + 8 * j, g = k / gs;
            const float s = s_s[r * G + g];
            const int z = s_z[r * G + g];
            const f32x4 va = *reinterpret_cast<const f32x4 *>(row + k);
            const f32x4 vb = *reinterpret_cast<const f32x4 *>(row + k + 4);
            const float w[8] = {va[0], va[1], va[2], va[3], vb[0], vb[1], vb[2], vb[3]};
            uint32_t qv[8];
#pragma unroll
            for (int cidx = 0; cidx < 8; ++cidx) {
                int q = (int)rintf(__fdiv_rn(w[cidx], s)) + z;
                q = q < 0 ? 0 : (q > qmax ? qmax : q);
                qv[cidx] = (uint32_t)q;
            }
            if constexpr (BITS == 4) {
                uint32_t word = 0;
#pragma unroll
                for (int cidx = 0; cidx < 8; ++cidx) word |= qv[cidx] << (4 * (cidx / 2 + 4 * (cidx % 2)));
                s_out[j * 8 + r] = word;
            } else {
                // stage the raw codes, one byte each: [block j][channel r][feature]
                s_out[(j * 8 + r) * 2] = qv[0] | (qv[1] << 8) | (qv[2] << 16) | (qv[3] << 24);
                s_out[(j * 8 + r) * 2 + 1] = qv[4] | (qv[5] << 8) | (qv[6] << 16) | (qv[7] << 24);
            }
        }
        __syncthreads();
        if (tid < nb * WPB) {
            uint32_t word;
            if constexpr (BITS == 4) {
                word = s_out[tid];
            } else {
                const uint8_t *codes = reinterpret_cast<const uint8_t *>(s_out) + (tid / 6) * 64;   // [8][8]
                const int wi = tid % 6, m = wi >> 1, par = wi & 1;
                word = 0;
#pragma unroll
                for (int f = 0; f < 5; ++f) {
                    const int u = 5 * m + f;
                    if (u < 15) {
                        const int ch = 2 * (u >> 2) + par, pr = u & 3;
                        word |= (uint32_t)codes[ch * 8 + 2 * pr] << (3 * f);
                        word |= (uint32_t)codes[ch * 8 + 2 * pr + 1] << (16 + 3 * f);
                    }
                }
                word |= (uint32_t)((codes[(6 + par) * 8 + 6] >> m) & 1u) << 15;
                word |= (uint32_t)((codes[(6 + par) * 8 + 7] >> m) & 1u) << 31;
            }
            const int kb = k0 / 8 + tid / WPB;
            packed[(out_row + (size_t)(kb >> 2) * 64 + (kb & 3)) * WPB + tid % WPB] = word;
        }
        __syncthreads();
    }
}

}  // namespace

hipError_t launch_quantize(const float *W0, int N, int K, int bits, int group, uint32_t *packed, float *s0,
                           uint8_t *z0, hipStream_t stream)
{
    const int gs = group > 0 ? group : K, G = K / gs;
    const size_t smem = (size_t)16 * G * 4 + 2048;
    trace_before(KID_QUANTIZE, stream);
    if (bits == 4)
        hipLaunchKernelGGL(quantize_kernel<4>, dim3(N / 8), dim3(256), smem, stream, W0, K, gs, G, packed, s0, z0);
    else
        hipLaunchKernelGGL(quantize_kernel<3>, dim3(N / 8), dim3(256), smem, stream, W0, K, gs, G, packed, s0, z0);
    trace_after(KID_QUANTIZE, stream);
    return hipGetLastError();
}

}  // namespace peqa
