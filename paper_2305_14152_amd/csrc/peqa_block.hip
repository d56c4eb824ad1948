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
    size_t rs[PEQA_MAX_BLOCK];       // row sums of distinct input i (per-channel items, T > 16)
    size_t dys[PEQA_MAX_BLOCK];      // backward, per-channel item j: bf16(dY (s0 + ds)) [T, N]
    size_t crow[PEQA_MAX_BLOCK];     //   its row factors [T]
    size_t partial[PEQA_MAX_BLOCK];  //   per-token-tile partials of its scale gradient [tiles_t, N]
    size_t item;                     // scratch of one group-wise item at a time (the largest single need)
    size_t total;
};

BlockSpace carve_block(int32_t n, const peqa_block_item *items, int32_t T, int32_t op)
{
    BlockSpace w{};
    int xi[PEQA_MAX_BLOCK], ks[PEQA_MAX_BLOCK];
    const uint16_t *xs[PEQA_MAX_BLOCK];
    const int nx = distinct_inputs(n, items, xi, xs, ks);
    const size_t tiles_t = ((size_t)T + 127) / 128;
    size_t off = 0;
    for (int i = 0; i < nx; ++i) { w.rs[i] = off; off += round256((size_t)T * 2 * sizeof(float)); }
    size_t need = 0;
    for (int j = 0; j < n; ++j) {
        const peqa_layout *L = &items[j].layout;
        if (grouped(L)) {
            const size_t b = peqa_workspace_bytes(L, T, op);
            need = b > need ? b : need;
        } else if (op == PEQA_OP_BWD) {
            const size_t N = (size_t)L->n_out;
            w.dys[j] = off;     off += round256((size_t)T * N * sizeof(uint16_t));
            w.crow[j] = off;    off += round256((size_t)T * sizeof(float));
            w.partial[j] = off; off += round256(tiles_t * N * sizeof(float));
        }
    }
    w.item = off;
    w.total = off + round256(need);
    if (w.total == 0) w.total = 256;
    return w;
}

// Jobs of a multi-contraction launch in order of falling contraction length.
void sort_jobs(peqa::MultiArgs &m)
{
    for (int i = 1; i < m.n_jobs; ++i)
        for (int k = i; k > 0 && m.job[k].a.KC > m.job[k - 1].a.KC; --k) {
            const peqa::MultiJob t = m.job[k];
            m.job[k] = m.job[k - 1];
            m.job[k - 1] = t;
        }
}

// Auxiliary workgroups of a multi-contraction launch: after the first round of tiles (two per compute unit), a
// multiple of 8.
void place_aux(peqa::MultiArgs &m, int aux_wgs)
{
    int total = 0;
    for (int j = 0; j < m.n_jobs; ++j) total += peqa::gemm_multi_wgs(m.job[j].a.tiles_t, m.job[j].a.tiles_c);
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    const int first_round = 2 * cus / 8 * 8;
    m.aux_begin = total < first_round ? total : first_round;
    m.aux_wgs = (m.n_sdy > 0 || m.n_red > 0) ? aux_wgs : 0;
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
    // row sums of every distinct input of the per-channel items: one launch
    const float *rs[PEQA_MAX_BLOCK];
    if (nx > 0) {
        peqa::RowsumMulti r{};
        for (int i = 0; i < peqa::ROWSUM_MAX; ++i) {
            const int k = i < nx ? i : nx - 1;
            float *dst = reinterpret_cast<float *>(ws + w.rs[k]);
            for (int j = 0; j < n; ++j)
                if (xi[j] == k && items[j].row_sums) { dst = items[j].row_sums; break; }
            r.X[i] = xs[k]; r.K[i] = ks[k]; r.rs[i] = dst;
            if (i < nx) rs[i] = dst;
        }
        r.n = nx; r.T = T;
        if (peqa::launch_rowsum_multi(r, s) != hipSuccess) return PEQA_ERR_DEVICE;
    }
    // all per-channel contractions: one launch
    peqa::MultiArgs m{};
    for (int j = 0; j < n; ++j) {
        const peqa_block_item &it = items[j];
        if (grouped(&it.layout)) continue;
        const int N = it.layout.n_out, K = it.layout.k_in;
        peqa::MultiJob &job = m.job[m.n_jobs++];
        job.mode = peqa::MODE_Y;
        peqa::GemmArgs &a = job.a;
        a.packed = it.packed; a.A = it.X; a.T = T; a.KC = K; a.C = N; a.K = K;
        a.tiles_c = (N + 255) / 256; a.tiles_t = (T + 127) / 128;
        a.s0 = it.s0; a.ds = it.ds; a.z0 = it.z0; a.rs = rs[xi[j]]; a.out = it.Y;
    }
    if (m.n_jobs > 0) {
        sort_jobs(m);
        place_aux(m, 0);
        if (peqa::launch_gemm_multi(items[0].layout.bits, m, s) != hipSuccess) return PEQA_ERR_DEVICE;
    }
    for (int j = 0; j < n; ++j) {
        const peqa_block_item &it = items[j];
        if (!grouped(&it.layout)) continue;
        st = peqa_linear_fwd(&it.layout, it.packed, it.s0, it.ds, it.z0, it.X, T, it.Y, ws + w.item,
                             workspace_bytes - w.item, stream);
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
    hipStream_t s = static_cast<hipStream_t>(stream);
    const BlockSpace w = carve_block(n, items, T, PEQA_OP_BWD);
    int xi[PEQA_MAX_BLOCK], ks[PEQA_MAX_BLOCK];
    const uint16_t *xs[PEQA_MAX_BLOCK];
    const int nx = distinct_inputs(n, items, xi, xs, ks);
    const int tiles_t = (T + 127) / 128;
    const int bits = items[0].layout.bits;

    // ---- per-channel items.  Row sums of the inputs whose scale gradient is wanted: the caller's (kept from the
    // forward), else taken here, all in one launch.
    const float *rs[PEQA_MAX_BLOCK] = {nullptr};
    {
        peqa::RowsumMulti r{};
        int nr = 0;
        for (int i = 0; i < nx; ++i) {
            bool wanted = false;
            const float *have = nullptr;
            for (int j = 0; j < n; ++j)
                if (xi[j] == i) {
                    wanted = wanted || items[j].d_ds != nullptr;
                    if (items[j].row_sums) have = items[j].row_sums;
                }
            if (have || !wanted) { rs[i] = have; continue; }
            float *dst = reinterpret_cast<float *>(ws + w.rs[i]);
            r.X[nr] = xs[i]; r.K[nr] = ks[i]; r.rs[nr] = dst;
            ++nr;
            rs[i] = dst;
        }
        if (nr > 0) {
            for (int i = nr; i < peqa::ROWSUM_MAX; ++i) { r.X[i] = r.X[nr - 1]; r.K[i] = r.K[nr - 1]; r.rs[i] = r.rs[nr - 1]; }
            r.n = nr; r.T = T;
            if (peqa::launch_rowsum_multi(r, s) != hipSuccess) return PEQA_ERR_DEVICE;
        }
    }
    // First launch: every scale-gradient contraction, and in its auxiliary workgroups the scaling of dY for every
    // dX contraction.  Second launch: every dX contraction, and the fixed-order sums of the first launch's partials.
    peqa::MultiArgs ma{}, mb{};
    int sdy_blocks = 0, red_chunks = 0;
    for (int j = 0; j < n; ++j) {
        const peqa_block_item &it = items[j];
        if (grouped(&it.layout)) continue;
        const int N = it.layout.n_out, K = it.layout.k_in;
        uint16_t *dys = reinterpret_cast<uint16_t *>(ws + w.dys[j]);
        float *crow = reinterpret_cast<float *>(ws + w.crow[j]);
        float *partial = reinterpret_cast<float *>(ws + w.partial[j]);
        if (it.d_ds) {
            peqa::MultiJob &job = ma.job[ma.n_jobs++];
            job.mode = peqa::MODE_DDS;
            peqa::GemmArgs &a = job.a;
            a.packed = it.packed; a.A = it.X; a.T = T; a.KC = K; a.C = N; a.K = K;
            a.tiles_c = (N + 255) / 256; a.tiles_t = tiles_t;
            a.z0 = it.z0; a.rs = rs[xi[j]]; a.dY = it.dY; a.partial = partial;
            peqa::ReduceJob &r = mb.red[mb.n_red++];
            r.partial = partial; r.out = it.d_ds; r.ntiles = tiles_t; r.n = N;
            red_chunks += (N + 255) / 256;
            r.chunk_end = red_chunks;
        }
        if (it.dX) {
            peqa::ScaleDyJob &sd = ma.sdy[ma.n_sdy++];
            sd.dY = it.dY; sd.s0 = it.s0; sd.ds = it.ds; sd.z0 = it.z0; sd.dYs = dys; sd.crow = crow; sd.T = T; sd.N = N;
            sdy_blocks += (T + peqa::SDY_ROWS_HOST - 1) / peqa::SDY_ROWS_HOST;
            sd.blk_end = sdy_blocks;
            peqa::MultiJob &job = mb.job[mb.n_jobs++];
            job.mode = peqa::MODE_DX;
            peqa::GemmArgs &a = job.a;
            a.packed = it.packed; a.A = dys; a.T = T; a.KC = N; a.C = K; a.K = K;
            a.tiles_c = (K + 255) / 256; a.tiles_t = tiles_t;
            a.crow = crow; a.out = it.dX;
        }
    }
    if (ma.n_jobs > 0 || ma.n_sdy > 0) {
        sort_jobs(ma);
        place_aux(ma, 128);
        if (peqa::launch_gemm_multi(bits, ma, s) != hipSuccess) return PEQA_ERR_DEVICE;
    }
    if (mb.n_jobs > 0 || mb.n_red > 0) {
        sort_jobs(mb);
        place_aux(mb, 64);
        if (peqa::launch_gemm_multi(bits, mb, s) != hipSuccess) return PEQA_ERR_DEVICE;
    }

    // ---- group-wise items, one by one
    for (int j = 0; j < n; ++j) {
        const peqa_block_item &it = items[j];
        if (!grouped(&it.layout)) continue;
        st = peqa_linear_bwd(&it.layout, it.packed, it.s0, it.ds, it.z0, it.X, it.dY, T, it.dX, it.d_ds, ws + w.item,
                             workspace_bytes - w.item, stream);
        if (st != PEQA_OK) return st;
    }
    return PEQA_OK;
}

}  // extern "C"
