// Eq. 1 of the paper: round-to-nearest asymmetric quantization with a min-max range,
// fused with the dense packing of the codes into 8x8 blocks (layout: peqa_bit_location()).
//
// One workgroup quantizes 8 output channels (one row of blocks).  Pass 1 reduces min/max
// per (channel, group) and derives s0, z0; pass 2 re-reads the rows (from L2), rounds,
// and assembles whole packed words in LDS so that they leave in runs of 4 blocks (a tile row).
// HBM-bound: 4 N K bytes in, N K b / 8 bytes out.
//
// Every fp32 step below is a single IEEE operation (correctly rounded divide, no fused
// multiply-add), because the codes must match the definition bit for bit.  The one divide per
// weight, w / s, is the exception in form only: it is taken as (float)((double)w * rs) with
// rs = 1.0 / (double)s formed once per scale by a correctly rounded fp64 divide.  That product is
// within 2^-52 (relative) of the true quotient, while the quotient of two fp32 numbers is never
// closer than 2^-49 (relative) to a point midway between two fp32 numbers (w - m s is a non-zero
// multiple of the last bit of a 49-bit product), so rounding it to fp32 gives the correctly
// rounded fp32 quotient: the same bits, at a third of the instructions (the correctly rounded fp32
// divide sequence made this kernel ALU-bound at 2.2 TB/s).
#include "peqa_device.h"
#include "peqa_kernels.h"

// No fused multiply-add anywhere in this file: every product below is rounded before it is added or
// subtracted, as the definition has it.  Products and differences are written with plain operators for
// that reason: the __fmul_rn / __fsub_rn spellings are header functions compiled outside this pragma,
// and the compiler fuses them (measured: scales one ulp off the definition).
#pragma clang fp contract(off)

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
            const float range = xmax - xmin;
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
            const double rs = 1.0 / (double)s;
            const int z = s_z[r * G + g];
            const f32x4 va = *reinterpret_cast<const f32x4 *>(row + k);
            const f32x4 vb = *reinterpret_cast<const f32x4 *>(row + k + 4);
            const float w[8] = {va[0], va[1], va[2], va[3], vb[0], vb[1], vb[2], vb[3]};
            uint32_t qv[8];
#pragma unroll
            for (int cidx = 0; cidx < 8; ++cidx) {
                int q = (int)rintf((float)((double)w[cidx] * rs)) + z;
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

// The same quantizer with the eight rows of a workgroup held in registers between the range pass and
// the code pass, so that W0 is read from memory once: 1024 threads, 128 per channel row, thread
// (r, l) keeps the 4-float vectors l, l + 128, ... (NV of them) of row r.  Arithmetic per element is
// that of quantize_kernel, operation for operation.  Serves K <= 512 NV.
//
// SEARCH: the error-minimising initialisation of Sec. 3.2 over a grid of clipped ranges.  For ratio
// r_j = 1 - j * step (j = 0 .. n_ratios - 1; r_0 = 1 is Eq. 1 as it stands) the range of every
// (channel, group) becomes [r_j xmin, r_j xmax]; the candidate with the smallest
// sum_k (w - s (Q - z))^2 is kept (the first of equal ones).  Residuals are formed in fp32 (one
// multiply, one subtract), squared and summed in fp64: 16 lanes by shuffles, then the 64-feature
// segments of a group in order, so the result does not depend on timing.
template <int BITS, int NV, bool SEARCH>
__global__ __launch_bounds__(1024) void quantize_resident_kernel(const float *__restrict__ W0, int K, int gs, int G,
                                                                  uint32_t *__restrict__ packed,
                                                                  float *__restrict__ s0, uint8_t *__restrict__ z0,
                                                                  int n_ratios, float step)
{
    extern __shared__ __align__(16) uint8_t smem[];
    // [8][G] each: bits of max(w, 0), bits of max(-w, 0) (non-negative floats order like their bit
    // patterns, so the range reduction is an integer max: exact and order-free), then s and z
    uint32_t *s_max = reinterpret_cast<uint32_t *>(smem);
    uint32_t *s_neg = s_max + 8 * G;
    float *s_s = reinterpret_cast<float *>(s_neg + 8 * G);
    int *s_z = reinterpret_cast<int *>(s_s + 8 * G);
    double *s_rs = reinterpret_cast<double *>(s_z + 8 * G);             // [8][G] 1 / s in fp64
    uint32_t *s_codes = reinterpret_cast<uint32_t *>(s_rs + 8 * G);      // [8][K / 4] words = one byte per code
    // SEARCH only: the best candidate so far per (channel, group), and the error sums per 64-feature segment
    double *b_err = reinterpret_cast<double *>(s_codes + 2 * K);        // [8][G]
    double *b_rs = b_err + 8 * G;
    double *seg_err = b_rs + 8 * G;                                     // [8][K / 64]
    float *b_s = reinterpret_cast<float *>(seg_err + (K >> 3));
    int *b_z = reinterpret_cast<int *>(b_s + 8 * G);

    constexpr int qmax = (1 << BITS) - 1;
    constexpr int WPB = 2 * BITS;
    const int tid = threadIdx.x, r = tid >> 7, l = tid & 127;
    const int ib = blockIdx.x;
    const int K4 = K >> 2;
    const f32x4 *row = reinterpret_cast<const f32x4 *>(W0 + (size_t)(ib * 8 + r) * K);

    f32x4 v[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int k4 = l + 128 * i;
        v[i] = k4 < K4 ? row[k4] : f32x4{0.f, 0.f, 0.f, 0.f};      // zeros are neutral: the range always holds 0
    }
    for (int e = tid; e < 16 * G; e += 1024) s_max[e] = 0u;          // s_max and s_neg
    __syncthreads();

    // ---- range per (channel, group): 16 lanes hold 64 consecutive features, always of one group
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        float xmax = 0.f, xneg = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (v[i][e] > xmax) xmax = v[i][e];
            if (-v[i][e] > xneg) xneg = -v[i][e];
        }
#pragma unroll
        for (int o = 8; o >= 1; o >>= 1) {
            const float a = __shfl_xor(xmax, o), b = __shfl_xor(xneg, o);
            if (a > xmax) xmax = a;
            if (b > xneg) xneg = b;
        }
        const int k4 = l + 128 * i;
        if ((l & 15) == 0 && k4 < K4) {
            const int g = (4 * k4) / gs;
            atomicMax(&s_max[r * G + g], __float_as_uint(xmax));
            atomicMax(&s_neg[r * G + g], __float_as_uint(xneg));
        }
    }
    __syncthreads();
    // (s, z, 1 / s) of candidate j for entry e = r * G + g
    auto candidate = [&](int e, int j) {
        const float xmax = __uint_as_float(s_max[e]);
        const float xneg = __uint_as_float(s_neg[e]);
        float xmin = xneg > 0.f ? -xneg : 0.f;
        float hi = xmax;
        if constexpr (SEARCH) {
            const float jstep = (float)j * step;
            const float ratio = 1.f - jstep;
            xmin = ratio * xmin;
            hi = ratio * hi;
        }
        const float range = hi - xmin;
        float s = __fdiv_rn(range, (float)qmax);
        int z;
        if (!(s > 0.f)) {
            s = 1.f;
            z = 0;
        } else {
            z = (int)rintf(__fdiv_rn(-xmin, s));
            z = z < 0 ? 0 : (z > qmax ? qmax : z);
        }
        s_s[e] = s;
        s_z[e] = z;
        s_rs[e] = 1.0 / (double)s;
    };
    for (int e = tid; e < 8 * G; e += 1024) candidate(e, 0);
    __syncthreads();
    if constexpr (SEARCH) {
        const int segs = K >> 6, per = gs >> 6;                          // segments per row / per group
        for (int j = 0; j < n_ratios; ++j) {
            // squared residuals of candidate j, this thread's vectors, summed over 16 lanes = one segment
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const int k4 = l + 128 * i;
                double err = 0.0;
                if (k4 < K4) {
                    const int g = (4 * k4) / gs;
                    const float sc = s_s[r * G + g];
                    const double rs = s_rs[r * G + g];
                    const int z = s_z[r * G + g];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        int q = (int)rintf((float)((double)v[i][e] * rs)) + z;
                        q = q < 0 ? 0 : (q > qmax ? qmax : q);
                        const float back = sc * (float)(q - z);
                        const float d = v[i][e] - back;
                        err += (double)d * (double)d;
                    }
                }
#pragma unroll
                for (int o = 8; o >= 1; o >>= 1) err += __shfl_xor(err, o);
                if ((l & 15) == 0 && k4 < K4) seg_err[r * segs + (k4 >> 4)] = err;
            }
            __syncthreads();
            for (int e = tid; e < 8 * G; e += 1024) {
                const int rr = e / G, g = e - rr * G;
                double err = 0.0;
                for (int q = 0; q < per; ++q) err += seg_err[rr * segs + g * per + q];
                if (j == 0 || err < b_err[e]) {
                    b_err[e] = err;
                    b_s[e] = s_s[e];
                    b_z[e] = s_z[e];
                    b_rs[e] = s_rs[e];
                }
                if (j + 1 < n_ratios) {
                    candidate(e, j + 1);
                } else {
                    s_s[e] = b_s[e];
                    s_z[e] = b_z[e];
                    s_rs[e] = b_rs[e];
                }
            }
            __syncthreads();
        }
    }
    for (int e = tid; e < 8 * G; e += 1024) {
        const int rr = e / G, g = e - rr * G;
        s0[(size_t)(ib * 8 + rr) * G + g] = s_s[e];
        z0[(size_t)(ib * 8 + rr) * G + g] = (uint8_t)s_z[e];
    }

    // ---- codes of all eight rows into LDS (one byte per code, [8][K]), then the packed words
    const size_t out_row = (size_t)(ib / 16) * (K / 32) * 64 + (size_t)(ib % 16) * 4;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int k4 = l + 128 * i;
        if (k4 < K4) {
            const int g = (4 * k4) / gs;
            const double rs = s_rs[r * G + g];
            const int z = s_z[r * G + g];
            uint32_t w = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                int q = (int)rintf((float)((double)v[i][e] * rs)) + z;
                q = q < 0 ? 0 : (q > qmax ? qmax : q);
                w |= (uint32_t)q << (8 * e);
            }
            s_codes[r * K4 + k4] = w;
        }
    }
    __syncthreads();
    const int nwords = (K >> 3) * WPB;                               // packed words of this row of blocks
    for (int e = tid; e < nwords; e += 1024) {
        const int kb = e / WPB, wi = e % WPB;
        uint32_t word = 0;
        if constexpr (BITS == 4) {
            // word wi = channel wi of the block: nibble cc / 2 + 4 (cc % 2) holds feature cc
            const uint32_t lo = s_codes[wi * K4 + 2 * kb], hi = s_codes[wi * K4 + 2 * kb + 1];
#pragma unroll
            for (int cc = 0; cc < 8; ++cc) {
                const uint32_t q = ((cc < 4 ? lo : hi) >> (8 * (cc & 3))) & 0xFFu;
                word |= q << (4 * (cc / 2 + 4 * (cc % 2)));
            }
        } else {
            const uint8_t *codes = reinterpret_cast<const uint8_t *>(s_codes);   // [8][K]
            const int m = wi >> 1, par = wi & 1;
            auto code = [&](int ch, int cc) { return (uint32_t)codes[(size_t)ch * K + 8 * kb + cc]; };
#pragma unroll
            for (int f = 0; f < 5; ++f) {
                const int u = 5 * m + f;
                if (u < 15) {
                    const int ch = 2 * (u >> 2) + par, pr = u & 3;
                    word |= code(ch, 2 * pr) << (3 * f);
                    word |= code(ch, 2 * pr + 1) << (16 + 3 * f);
                }
            }
            word |= ((code(6 + par, 6) >> m) & 1u) << 15;
            word |= ((code(6 + par, 7) >> m) & 1u) << 31;
        }
        packed[(out_row + (size_t)(kb >> 2) * 64 + (kb & 3)) * WPB + wi] = word;
    }
}

constexpr int kMaxDevQ = 64;
}  // namespace
bool quantize_resident_fits(int K, int G, bool search);
namespace {

// dynamic LDS of quantize_resident_kernel
size_t resident_lds(int K, int G, bool search) { return (size_t)(search ? 384 : 192) * G + (size_t)(search ? 9 : 8) * K; }

template <int BITS, int NV, bool SEARCH>
hipError_t launch_resident(const float *W0, int N, int K, int gs, int G, uint32_t *packed, float *s0, uint8_t *z0,
                           int n_ratios, float step, hipStream_t stream)
{
    static int attr_bytes[kMaxDevQ];                                  // dynamic LDS allowed so far, per device
    const size_t smem = resident_lds(K, G, SEARCH);
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevQ) return hipErrorInvalidDevice;
    if (smem > 48 * 1024 && (int)smem > attr_bytes[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(quantize_resident_kernel<BITS, NV, SEARCH>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_bytes[dev] = (int)smem;
    }
    hipLaunchKernelGGL((quantize_resident_kernel<BITS, NV, SEARCH>), dim3(N / 8), dim3(1024), smem, stream, W0, K, gs, G,
                       packed, s0, z0, n_ratios, step);
    return hipSuccess;
}

// true if a register-resident instantiation took the call (K <= 12288 and the LDS need fits)
template <int BITS, bool SEARCH>
bool launch_resident_for(const float *W0, int N, int K, int gs, int G, uint32_t *packed, float *s0, uint8_t *z0,
                         int n_ratios, float step, hipStream_t stream, hipError_t *err)
{
    if (!quantize_resident_fits(K, G, SEARCH)) return false;
    const int nv = (K + 511) / 512;
    if (nv <= 8) *err = launch_resident<BITS, 8, SEARCH>(W0, N, K, gs, G, packed, s0, z0, n_ratios, step, stream);
    else if (nv <= 16) *err = launch_resident<BITS, 16, SEARCH>(W0, N, K, gs, G, packed, s0, z0, n_ratios, step, stream);
    else *err = launch_resident<BITS, 24, SEARCH>(W0, N, K, gs, G, packed, s0, z0, n_ratios, step, stream);
    return true;
}

}  // namespace

hipError_t launch_quantize(const float *W0, int N, int K, int bits, int group, uint32_t *packed, float *s0,
                           uint8_t *z0, hipStream_t stream)
{
    const int gs = group > 0 ? group : K, G = K / gs;
    const size_t smem = (size_t)16 * G * 4 + 2048;
    trace_before(KID_QUANTIZE, stream);
    // rows up to 12288 features stay in registers between the two passes; longer ones are read twice
    hipError_t err = hipSuccess;
    const bool resident = bits == 4 ? launch_resident_for<4, false>(W0, N, K, gs, G, packed, s0, z0, 1, 0.f, stream, &err)
                                    : launch_resident_for<3, false>(W0, N, K, gs, G, packed, s0, z0, 1, 0.f, stream, &err);
    if (resident) {
        if (err != hipSuccess) return err;
    } else if (bits == 4)
        hipLaunchKernelGGL(quantize_kernel<4>, dim3(N / 8), dim3(256), smem, stream, W0, K, gs, G, packed, s0, z0);
    else
        hipLaunchKernelGGL(quantize_kernel<3>, dim3(N / 8), dim3(256), smem, stream, W0, K, gs, G, packed, s0, z0);
    trace_after(KID_QUANTIZE, stream);
    return hipGetLastError();
}

bool quantize_resident_fits(int K, int G, bool search)
{
    return K <= 12288 && resident_lds(K, G, search) <= 150 * 1024;
}

hipError_t launch_quantize_search(const float *W0, int N, int K, int bits, int group, int n_ratios, float step,
                                  uint32_t *packed, float *s0, uint8_t *z0, hipStream_t stream)
{
    const int gs = group > 0 ? group : K, G = K / gs;
    hipError_t err = hipSuccess;
    trace_before(KID_QUANTIZE, stream);
    const bool done = bits == 4 ? launch_resident_for<4, true>(W0, N, K, gs, G, packed, s0, z0, n_ratios, step, stream, &err)
                                : launch_resident_for<3, true>(W0, N, K, gs, G, packed, s0, z0, n_ratios, step, stream, &err);
    trace_after(KID_QUANTIZE, stream);
    if (!done) return hipErrorInvalidValue;
    return err != hipSuccess ? err : hipGetLastError();
}

}  // namespace peqa
