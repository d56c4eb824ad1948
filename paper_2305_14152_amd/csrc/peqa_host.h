// Host-side helpers shared by the files that implement the C-ABI (peqa_api.hip, peqa_block.hip).
#pragma once

#include "../../include/peqa.h"
#include "peqa_kernels.h"

namespace peqa {
namespace host {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round256(size_t b) { return (b + 255) & ~(size_t)255; }
inline int groups(const peqa_layout *L) { return L->group_size > 0 ? L->k_in / L->group_size : 1; }
// A single group per channel is the per-channel layer, and takes its kernels.
inline bool grouped(const peqa_layout *L) { return groups(L) > 1; }
inline peqa_status dev_status(hipError_t e) { return e == hipSuccess ? PEQA_OK : PEQA_ERR_DEVICE; }

// Contraction index at which the second half of a contraction of length n starts: the contraction
// kernels give each of their two wave groups one half (n % 128 == 0, so both are whole steps of 64),
// and the row sums their epilogues use are taken over the same halves.
inline int split_point(int n) { return n / 2; }

constexpr int GEMV_MAX_T = 16;   // forward calls with at most this many tokens take the matrix-vector path

// One layer of a matrix-vector launch (validated by the caller).
struct GemvItem {
    const peqa_layout *L;
    const uint32_t *packed;
    const float *s0, *ds;
    const uint8_t *z0;
    const float *dz;
    const uint16_t *X;
    uint16_t *Y;
};
// Slices per layer: `block_plan` balances layers of different shapes against each other (peqa_block_fwd);
// otherwise all layers share K and take the slicing of one layer of their summed channels.
// `zbyte`: no item has a trained zero-point offset (dz), which allows longer slices of group-wise layers.
void gemv_slicing(int n, const GemvItem *items, int32_t T, bool block_plan, bool zbyte, int *S);
// fp32 partials of the sliced layers of such a launch
size_t gemv_partial_bytes(int n, const GemvItem *items, int32_t T, bool block_plan, bool zbyte);
// One matrix-vector launch (plus the sum of the slices, if any) for n <= GEMV_MAX_LAYERS layers of one bit width.
peqa_status gemv_forward(int n, const GemvItem *items, int32_t T, bool block_plan, float *partial, hipStream_t s);

}  // namespace host
}  // namespace peqa
