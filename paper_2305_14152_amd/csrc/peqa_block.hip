// Block-level entry points of the C-ABI (include/peqa.h): the linears of a decoder block -- any list of up to
// PEQA_MAX_BLOCK independent PEQA layers, each with its own input -- behind one forward and one backward call.
#include "peqa_host.h"

using namespace peqa::host;

namespace {

peqa_status check_items(int32_t n, const peqa_block_item *items, int32_t T)
{
    if (!items) return PEQA_ERR_NULL;
    if (n < 1 || n > PEQA_MAX_BLOCK) return PEQA_ERR_PARAM;
    if (T < 1 || T > (1 << 24)) return PEQA_ERR_SHAPE;
    for (int j = 0; j < n; ++j) {
        const peqa_status st = peqa_check_layout(&items[j].layout);
        if (st != PEQA_OK) return st;
        if (items[j].layout.bits != items[0].layout.bits) return PEQA_ERR_PARAM;
    }
    return PEQA_OK;
}

// Distinct inputs of the per-channel items, in order of first appearance: xi[j] = index of item j's input.
int distinct_inputs(int32_t n, const peqa_block_item *items, int *xi, const uint16_t **xs, int *ks)
{
    int nx = 0;
    for (int j = 0; j < n; ++j) {
        xi[j] = -1;
        if (grouped(&items[j].layout)) continue;
        for (int i = 0; i < nx; ++i)
            if (xs[i] == items[j].X && ks[i] == items[j].layout.k_in) xi[j] = i;
        if (xi[j] < 0) {
            xs[nx] = items[j].X;
            ks[nx] = items[j].layout.k_in;
            xi[j] = nx++;
        }
    }
    return nx;
}

struct BlockSpace {
    size_t rs[PEQA_MAX_BLOCK];     // row sums of distinct input i (per-channel items, T > 16)
    size_t item;                   // scratch of one item at a time (the largest single need)
    size_t total;
};

BlockSpace carve_block(int32_t n, const peqa_block_item *items, int32_t T, int32_t op)
{
    BlockSpace w{};
    int xi[PEQA_MAX_BLOCK], ks[PEQA_MAX_BLOCK];
    const uint16_t *xs[PEQA_MAX_BLOCK];
    const int nx = distinct_inputs(n, items, xi, xs, ks);
    size_t off = 0;
    for (int i = 0; i < nx; ++i) { w.rs[i] = off; off += round256((size_t)T * 2 * sizeof(float)); }
    w.item = off;
    size_t need = 0;
    for (int j = 0; j < n; ++j) {
        const size_t b = peqa_workspace_bytes(&items[j].layout, T, op);
        need = b > need ? b : need;
    }
    w.total = off + round256(need);
    return w;
}

}  // namespace

extern "C" {

size_t peqa_block_workspace_bytes(int32_t n, const peqa_block_item *items, int32_t T, int32_t op)
{
    if (check_items(n, items, T) != PEQA_OK) return 0;
    if (op != PEQA_OP_FWD && op != PEQA_OP_BWD) return 0;
    if (op == PEQA_OP_FWD && T <= GEMV_MAX_T) {
        GemvItem gi[PEQA_MAX_BLOCK];
        for (int j = 0; j < n; ++j) gi[j] = GemvItem{&items[j].layout, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
        const size_t b = round256(gemv_partial_bytes(n, gi, T, true, true));
        return b ? b : 256;
    }
    return carve_block(n, items, T, op).total;
}

peqa_status peqa_block_fwd(int32_t n, const peqa_block_item *items, int32_t T, void *workspace,
                           size_t workspace_bytes, void *stream)
{
    peqa_status st = check_items(n, items, T);
    if (st != PEQA_OK) return st;
    for (int j = 0; j < n; ++j) {
        const peqa_block_item &it = items[j];
        if (!it.packed || !it.s0 || !it.z0 || !it.X || !it.Y) return PEQA_ERR_NULL;
        if (!aligned16(it.packed) || !aligned16(it.s0) || !aligned16(it.z0) || !aligned16(it.X) || !aligned16(it.Y) ||
            (it.ds && !aligned16(it.ds)) || (it.row_sums && !aligned16(it.row_sums)))
            return PEQA_ERR_ALIGN;
    }
    const size_t need = peqa_block_workspace_bytes(n, items, T, PEQA_OP_FWD);
    if (!workspace || workspace_bytes < need) return PEQA_ERR_WORKSPACE;
    if (!aligned16(workspace)) return PEQA_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t *ws = static_cast<uint8_t *>(workspace);

    if (T <= GEMV_MAX_T) {
        GemvItem gi[PEQA_MAX_BLOCK];
        for (int j = 0; j < n; ++j)
            gi[j] = GemvItem{&items[j].layout, items[j].packed, items[j].s0, items[j].ds, items[j].z0, nullptr,
                             items[j].X, items[j].Y};
        return gemv_forward(n, gi, T, true, reinterpret_cast<float *>(ws), s);
    }

    const BlockSpace w = carve_block(n, items, T, PEQA_OP_FWD);
    int xi[PEQA_MAX_BLOCK], ks[PEQA_MAX_BLOCK];
    const uint16_t *xs[PEQA_MAX_BLOCK];
    const int nx = distinct_inputs(n, items, xi, xs, ks);
    const float *rs[PEQA_MAX_BLOCK];
    for (int i = 0; i < nx; ++i) {
        float *dst = reinterpret_cast<float *>(ws + w.rs[i]);
        for (int j = 0; j < n; ++j)
            if (xi[j] == i && items[j].row_sums) { dst = items[j].row_sums; break; }
        if (peqa::launch_rowsum(xs[i], T, ks[i], split_point(ks[i]), dst, s) != hipSuccess) return PEQA_ERR_DEVICE;
        rs[i] = dst;
    }
    for (int j = 0; j < n; ++j) {
        const peqa_block_item &it = items[j];
        if (grouped(&it.layout)) {
            st = peqa_linear_fwd(&it.layout, it.packed, it.s0, it.ds, it.z0, it.X, T, it.Y, ws + w.item,
                                 workspace_bytes - w.item, stream);
        } else {
            peqa_fwd_item one{it.layout, it.packed, it.s0, it.ds, it.z0, it.Y};
            st = peqa_linear_fwd_fused_rs(1, &one, it.X, rs[xi[j]], T, ws + w.item, workspace_bytes - w.item, stream);
        }
        if (st != PEQA_OK) return st;
    }
    return PEQA_OK;
}

peqa_status peqa_block_bwd(int32_t n, const peqa_block_item *items, int32_t T, void *workspace,
                           size_t workspace_bytes, void *stream)
{
    peqa_status st = check_items(n, items, T);
    if (st != PEQA_OK) return st;
    for (int j = 0; j < n; ++j) {
        const peqa_block_item &it = items[j];
        if (!it.packed || !it.s0 || !it.z0 || !it.dY) return PEQA_ERR_NULL;
        if (it.d_ds && !it.X) return PEQA_ERR_NULL;
        if (!aligned16(it.packed) || !aligned16(it.s0) || !aligned16(it.z0) || !aligned16(it.dY) ||
            (it.X && !aligned16(it.X)) || (it.ds && !aligned16(it.ds)) || (it.dX && !aligned16(it.dX)) ||
            (it.d_ds && !aligned16(it.d_ds)) || (it.row_sums && !aligned16(it.row_sums)))
            return PEQA_ERR_ALIGN;
    }
    const size_t need = peqa_block_workspace_bytes(n, items, T, PEQA_OP_BWD);
    if (!workspace || workspace_bytes < need) return PEQA_ERR_WORKSPACE;
    if (!aligned16(workspace)) return PEQA_ERR_ALIGN;
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    const BlockSpace w = carve_block(n, items, T, PEQA_OP_BWD);
    for (int j = 0; j < n; ++j) {
        const peqa_block_item &it = items[j];
        st = peqa_linear_bwd_rs(&it.layout, it.packed, it.s0, it.ds, it.z0, it.X, it.row_sums, it.dY, T, it.dX, it.d_ds,
                                ws + w.item, workspace_bytes - w.item, stream);
        if (st != PEQA_OK) return st;
    }
    return PEQA_OK;
}

}  // extern "C"
