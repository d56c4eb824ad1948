// Device-side helpers shared by the gfx950 kernels of the PEQA library:
// vector types for MFMA operands, bf16 <-> fp32 bit tricks, and the in-register
// unpacking of packed 3/4-bit codes into bf16 MFMA operand fragments.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace peqa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Codes are turned into bf16 without any int->float conversion: a b-bit code q placed
// in mantissa bits 3.. of the bf16 pattern of 16.0 (0x4180) denotes exactly 16 + q.
// Kernels contract against 16 + Q and take the constant offset (and the zero-point)
// out afterwards through row sums of the other operand.
constexpr float kCodeOffset = 16.0f;
constexpr uint32_t kMagic = 0x41804180u;   // two bf16 16.0
constexpr uint32_t kMask4 = 0x00780078u;   // 4-bit field at bits 3..6 of each half-word
constexpr uint32_t kMask3 = 0x00380038u;   // 3-bit field at bits 3..5 of each half-word

__device__ __forceinline__ float bf16_bits_to_float(uint32_t h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pair) { return __uint_as_float(pair & 0xFFFF0000u); }

// fp32 -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    return float_to_bf16_bits(lo) | (float_to_bf16_bits(hi) << 16);
}

// A pair of bf16 (16 + code), scaled and shifted in fp32 and rounded once (to nearest even) back to a
// bf16 pair:  lo -> s_lo * lo + b_lo,  hi -> s_hi * hi + b_hi.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t scale_pair(uint32_t pair, float s_lo, float b_lo, float s_hi, float b_hi)
{
    f32x2 v;
    v[0] = __builtin_fmaf(__uint_as_float(pair << 16), s_lo, b_lo);
    v[1] = __builtin_fmaf(__uint_as_float(pair & 0xFFFF0000u), s_hi, b_hi);
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// A pair of bf16 times a pair of fp32 factors, rounded once (to nearest even) back to a bf16 pair.
__device__ __forceinline__ uint32_t mul_pair(uint32_t pair, float s_lo, float s_hi)
{
    f32x2 v;
    v[0] = __uint_as_float(pair << 16) * s_lo;
    v[1] = __uint_as_float(pair & 0xFFFF0000u) * s_hi;
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Two fp32 rounded (to nearest even) to a bf16 pair: one conversion instruction.
__device__ __forceinline__ uint32_t cvt_pair(float lo, float hi)
{
    f32x2 v;
    v[0] = lo;
    v[1] = hi;
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// c + a.lo * b.lo + a.hi * b.hi of two bf16 pairs, in fp32 (v_dot2c_f32_bf16).
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}

// ((x shifted) & mask) | magic in two VALU ops (one when no shift is needed).  mask rides the
// constant bus (SGPR), magic a VGPR.  Volatile assembly, shift included, so that the unpacking
// stays exactly where the caller interleaves it with matrix instructions.
__device__ __forceinline__ uint32_t and_or(uint32_t x, uint32_t mask, uint32_t magic)
{
    uint32_t d;
    asm volatile("v_and_or_b32 %0, %1, %2, %3" : "=v"(d) : "v"(x), "s"(mask), "v"(magic));
    return d;
}
__device__ __forceinline__ uint32_t shr_and_or(uint32_t x, uint32_t sh, uint32_t mask, uint32_t magic)
{
    uint32_t d;
    asm volatile("v_lshrrev_b32 %0, %1, %2\n\tv_and_or_b32 %0, %0, %3, %4"
                 : "=&v"(d) : "n"(sh), "v"(x), "s"(mask), "v"(magic));
    return d;
}
__device__ __forceinline__ uint32_t shl_and_or(uint32_t x, uint32_t sh, uint32_t mask, uint32_t magic)
{
    uint32_t d;
    asm volatile("v_lshlrev_b32 %0, %1, %2\n\tv_and_or_b32 %0, %0, %3, %4"
                 : "=&v"(d) : "n"(sh), "v"(x), "s"(mask), "v"(magic));
    return d;
}

// Field number F (of width b) of both half-words of v -> pair of bf16 (16 + code).
template <int BITS, int F>
__device__ __forceinline__ uint32_t field_pair(uint32_t v, uint32_t magic)
{
    constexpr uint32_t mask = BITS == 4 ? kMask4 : kMask3;
    constexpr int sh = BITS * F - 3;
    if constexpr (sh < 0) return shl_and_or(v, 3, mask, magic);
    else if constexpr (sh == 0) return and_or(v, mask, magic);
    else return shr_and_or(v, sh, mask, magic);
}

// The 3-bit cell that lives in the spare top bits (15 and 31) of three words.
__device__ __forceinline__ uint32_t spare_pair3(uint32_t v0, uint32_t v1, uint32_t v2, uint32_t magic)
{
    uint32_t t = shr_and_or(v0, 12, 0x00080008u, magic);
    t = shr_and_or(v1, 11, 0x00100010u, t);
    return shr_and_or(v2, 10, 0x00200020u, t);
}

// ---------------------------------------------------------------------------------
// One 8x8 block of codes (8 channels x 8 features; 2*BITS words) -> eight operand
// fragments of 8 bf16 (4 registers) each, produced one at a time so that callers can
// spread the unpacking between matrix instructions.
//
// Along features: fragment r = channel r, elements = features 0..7 in order
//   (the operand of a contraction over input features: forward, scale gradient).
// Along channels: fragment f = feature f, elements = channels 0..7 in order
//   (the operand of a contraction over output channels: dX).
// Layout of the block's words: see peqa_bit_location() in peqa.h.
// ---------------------------------------------------------------------------------
template <int BITS, bool ALONG_CH>
struct BlockUnpacker {
    static constexpr int WPB = 2 * BITS;
    uint32_t lo[4], hi[4];      // along channels: half-words of partner channels merged
    uint32_t w[WPB];

    __device__ __forceinline__ void prepare(const uint32_t *words)
    {
#pragma unroll
        for (int i = 0; i < WPB; ++i) w[i] = words[i];
        if constexpr (ALONG_CH) {
            // After the merge the low half-word belongs to the even channel of a partner pair and
            // the high half-word to the odd one, which is the element order of the fragment.
#pragma unroll
            for (int m = 0; m < BITS; ++m) {
                lo[m] = __builtin_amdgcn_perm(w[2 * m + 1], w[2 * m], 0x05040100u);
                hi[m] = __builtin_amdgcn_perm(w[2 * m + 1], w[2 * m], 0x07060302u);
            }
        }
    }

    // register J (0..3: elements 2J, 2J+1) of fragment I (0..7)
    template <int I, int J>
    __device__ __forceinline__ uint32_t frag_reg(uint32_t magic) const
    {
        if constexpr (!ALONG_CH) {
            if constexpr (BITS == 4) {
                return field_pair<4, J>(w[I], magic);
            } else {
                constexpr int par = I % 2, u = 4 * (I / 2) + J;
                if constexpr (u < 15) return field_pair<3, u % 5>(w[2 * (u / 5) + par], magic);
                else return spare_pair3(w[par], w[2 + par], w[4 + par], magic);
            }
        } else {
            constexpr bool odd = I & 1;             // odd features live in the high half-words
            constexpr int p = I >> 1;
            if constexpr (BITS == 4) {
                return field_pair<4, p>(odd ? hi[J] : lo[J], magic);
            } else {
                constexpr int u = 4 * J + p;
                if constexpr (u < 15) return field_pair<3, u % 5>(odd ? hi[u / 5] : lo[u / 5], magic);
                else return odd ? spare_pair3(hi[0], hi[1], hi[2], magic) : spare_pair3(lo[0], lo[1], lo[2], magic);
            }
        }
    }

    template <int I>
    __device__ __forceinline__ u32x4 frag(uint32_t magic) const
    {
        u32x4 f;
        f[0] = frag_reg<I, 0>(magic);
        f[1] = frag_reg<I, 1>(magic);
        f[2] = frag_reg<I, 2>(magic);
        f[3] = frag_reg<I, 3>(magic);
        return f;
    }
};

// Per-channel backward, the part of dY the dX contraction reads:  dYs[t,i] = bf16(dY[t,i] (s0 + ds)[i])  and
// crow[t] = sum_i dYs[t,i] (16 + z0[i] + dz[i])  (from the rounded dYs, so that it cancels the code offset of the
// contraction exactly), for the SDY_ROWS token rows of row block `blk`, by one workgroup of 256 threads
// (the per-channel parameters are read once per four rows).  `red` is 16 floats of LDS.
constexpr int SDY_ROWS = 4;
__device__ __forceinline__ void scale_dy_rows(const uint16_t *__restrict__ dY, const float *__restrict__ s0,
                                              const float *__restrict__ ds, const uint8_t *__restrict__ z0,
                                              const float *__restrict__ dz, int T, int N, uint16_t *__restrict__ dYs,
                                              float *__restrict__ crow, int blk, float *red)
{
    const int tid = threadIdx.x;
    const int t0 = blk * SDY_ROWS, rows = min(SDY_ROWS, T - t0);
    const int n8s = N >> 3;
    float acc[SDY_ROWS];
#pragma unroll
    for (int r = 0; r < SDY_ROWS; ++r) acc[r] = 0.f;
    for (int n8 = tid; n8 < n8s; n8 += 256) {
        u32x4 v[SDY_ROWS];                                 // rows past T re-read the last one and are dropped
#pragma unroll
        for (int r = 0; r < SDY_ROWS; ++r)
            v[r] = reinterpret_cast<const u32x4 *>(dY + (size_t)(t0 + min(r, rows - 1)) * N)[n8];
        const f32x4 sa = *reinterpret_cast<const f32x4 *>(s0 + 8 * n8);
        const f32x4 sb = *reinterpret_cast<const f32x4 *>(s0 + 8 * n8 + 4);
        float s[8] = {sa[0], sa[1], sa[2], sa[3], sb[0], sb[1], sb[2], sb[3]};
        if (ds) {
            const f32x4 da = *reinterpret_cast<const f32x4 *>(ds + 8 * n8);
            const f32x4 db = *reinterpret_cast<const f32x4 *>(ds + 8 * n8 + 4);
#pragma unroll
            for (int i = 0; i < 4; ++i) { s[i] += da[i]; s[4 + i] += db[i]; }
        }
        const u32x2 zz = *reinterpret_cast<const u32x2 *>(z0 + 8 * n8);
        float zo[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) zo[i] = kCodeOffset + (float)((zz[i >> 2] >> (8 * (i & 3))) & 0xFFu);
        if (dz) {
            const f32x4 za = *reinterpret_cast<const f32x4 *>(dz + 8 * n8);
            const f32x4 zb = *reinterpret_cast<const f32x4 *>(dz + 8 * n8 + 4);
#pragma unroll
            for (int i = 0; i < 4; ++i) { zo[i] += za[i]; zo[4 + i] += zb[i]; }
        }
#pragma unroll
        for (int r = 0; r < SDY_ROWS; ++r) {
            u32x4 o;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t lo = float_to_bf16_bits(bf16_lo(v[r][p]) * s[2 * p]);
                const uint32_t hi = float_to_bf16_bits(bf16_hi(v[r][p]) * s[2 * p + 1]);
                o[p] = lo | (hi << 16);
                acc[r] += bf16_bits_to_float(lo) * zo[2 * p] + bf16_bits_to_float(hi) * zo[2 * p + 1];
            }
            if (r < rows) reinterpret_cast<u32x4 *>(dYs + (size_t)(t0 + r) * N)[n8] = o;
        }
    }
#pragma unroll
    for (int r = 0; r < SDY_ROWS; ++r) {
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) acc[r] += __shfl_xor(acc[r], o);
        if ((tid & 63) == 0) red[r * 4 + (tid >> 6)] = acc[r];
    }
    __syncthreads();
    if (tid < rows) crow[t0 + tid] = (red[tid * 4] + red[tid * 4 + 1]) + (red[tid * 4 + 2] + red[tid * 4 + 3]);
}

// out[j] = partial[0][j] + partial[1][j] + ... in that order (deterministic).
__device__ __forceinline__ void reduce_partials_at(const float *__restrict__ partial, int ntiles, size_t n, size_t j,
                                                   float *__restrict__ out)
{
    if (j >= n) return;
    // eight loads in flight, added in tile order
    float s = 0.f;
    int tt = 0;
    for (; tt + 8 <= ntiles; tt += 8) {
        float p[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) p[u] = partial[(size_t)(tt + u) * n + j];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += p[u];
    }
    for (; tt < ntiles; ++tt) s += partial[(size_t)tt * n + j];
    out[j] = s;
}

// One 64 x 64 tile of the step-major transposed copy that the token contraction of group-wise layers reads:
// dst[t / 32][cc][t % 32] = src[t, cc] for t < T, 0 for T <= t < Tp, tile (bt, bc) of 64 tokens x 64 columns,
// by one workgroup of 256 threads through `tile`, 64 x 66 bf16 of LDS.  C % 64 == 0.
__device__ __forceinline__ void transpose_pad_tile(const uint16_t *__restrict__ src, int T, int C, uint16_t *__restrict__ dst,
                                                   int bt, int bc, uint16_t (*tile)[64 + 2])
{
    const int t0 = bt * 64, c0 = bc * 64;
    const int ch = threadIdx.x & 7;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int row = (threadIdx.x >> 3) + 32 * h, t = t0 + row;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (t < T) v = *reinterpret_cast<const u32x4 *>(src + (size_t)t * C + c0 + 8 * ch);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            tile[row][8 * ch + 2 * e] = (uint16_t)(v[e] & 0xFFFFu);
            tile[row][8 * ch + 2 * e + 1] = (uint16_t)(v[e] >> 16);
        }
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int cc = (threadIdx.x >> 3) + 32 * h;
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            o[e] = (uint32_t)tile[8 * ch + 2 * e][cc] | ((uint32_t)tile[8 * ch + 2 * e + 1][cc] << 16);
        const int t = t0 + 8 * ch;                        // 8 tokens of one 32-token step
        *reinterpret_cast<u32x4 *>(dst + ((size_t)(t >> 5) * C + c0 + cc) * 32 + (t & 31)) = o;
    }
}

// A piece of the kernel's argument block read at a run-time (wavefront-uniform) byte offset: scalar loads from the
// kernarg segment.  Indexing an array inside a by-value kernel argument with a run-time index would make the
// compiler keep a private copy of the whole argument in scratch memory; this reads the segment itself.
typedef uint32_t __attribute__((may_alias)) u32_alias;
template <class T>
__device__ __forceinline__ T kernarg_load(uint32_t byte_offset)
{
    static_assert(sizeof(T) % 4 == 0, "whole dwords");
    typedef const __attribute__((address_space(4))) u32_alias *cptr;
    const cptr p = (cptr)((const __attribute__((address_space(4))) char *)__builtin_amdgcn_kernarg_segment_ptr() + byte_offset);
    T out;
    u32_alias *o = reinterpret_cast<u32_alias *>(&out);
#pragma unroll
    for (int i = 0; i < (int)(sizeof(T) / 4); ++i) o[i] = p[i];
    return out;
}

// s_barrier alone: no implied wait on outstanding LDS or memory operations.
__device__ __forceinline__ void bare_barrier() { asm volatile("s_barrier" ::: "memory"); }

// D = A * B + C on one 16x16 tile with a 32-deep contraction (compiler-scheduled form).
__device__ __forceinline__ f32x4 mfma16(const u32x4 &a, const u32x4 &b, const f32x4 &c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// D += A * B on one 16x16 tile with a 32-deep contraction.  Issued as inline assembly with the
// accumulator tied to an AGPR tuple: with the builtin, this compiler keeps rotating part of a
// 256-register accumulator set through VGPRs on every loop iteration.  The hardware does not
// interlock a read of the result by a non-matrix instruction: callers must put at least 18 wait
// states (mfma_result_fence) between the last of these and the first such read.
__device__ __forceinline__ void mfma16_acc(f32x4 &acc, const u32x4 &a, const u32x4 &b)
{
    // volatile: keeps the source order of the matrix instructions among themselves and relative
    // to the DMA queueing and the result fence (the scalar/vector work around them is still free)
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// An accumulator tile copied from its AGPRs to VGPRs at this point of the program (volatile: the
// compiler would otherwise gather every such copy of a kernel at one place).
__device__ __forceinline__ f32x4 read_acc(const f32x4 &acc)
{
    f32x4 v;
    asm volatile("v_accvgpr_read_b32 %0, %4\n\tv_accvgpr_read_b32 %1, %5\n\tv_accvgpr_read_b32 %2, %6\n\tv_accvgpr_read_b32 %3, %7"
                 : "=v"(v[0]), "=v"(v[1]), "=v"(v[2]), "=v"(v[3])
                 : "a"(acc[0]), "a"(acc[1]), "a"(acc[2]), "a"(acc[3]));
    return v;
}
__device__ __forceinline__ void mfma_result_fence()
{
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
}

// Global -> LDS DMA of 16 bytes per lane: lane l's bytes land at lds_dst + 16 l.  The source
// is sbase (uniform) + voff (per lane).  Issued from inline assembly so that the compiler does not
// serialise the ring with a conservative vmcnt(0); completion is tracked by hand with wait_vmcnt().
__device__ __forceinline__ void dma16(uint32_t voff, const void *sbase, uint32_t lds_dst)
{
    // sbase is the same in every lane; saying so keeps it in scalar registers wherever the compiler cannot tell
    const uint64_t u = (uint64_t)(uintptr_t)sbase;
    const uint64_t ub = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(u >> 32)) << 32) |
                        (uint32_t)__builtin_amdgcn_readfirstlane((int)u);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(ub), "s"(lds_dst) : "memory");
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

}  // namespace peqa
