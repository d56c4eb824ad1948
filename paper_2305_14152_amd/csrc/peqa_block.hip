// Block-level entry points of the C-ABI (include/peqa.h): the linears of a decoder block -- any list of up to
// PEQA_MAX_BLOCK independent PEQA layers, each with its own input -- behind one forward and one backward call.
#include "peqa_host.h"

using namespace peqa::host;

// every table of a launch holds an entry per item of a call
static_assert(peqa::MULTI_MAX_JOBS >= PEQA_MAX_BLOCK && peqa::DW_MAX_JOBS >= PEQA_MAX_BLOCK && peqa::GT_MAX >= PEQA_MAX_BLOCK &&
                  peqa::ROWSUM_MAX >= PEQA_MAX_BLOCK && peqa::GEMV_MAX_LAYERS >= PEQA_MAX_BLOCK,
              "launch tables against PEQA_MAX_BLOCK");

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

// Distinct inputs of the items, in order of first appearance: xi[j] = index of item j's input.
int distinct_inputs(int32_t n, const peqa_block_item *items, int *xi, const uint16_t **xs, int *ks)
{
    int nx = 0;
    for (int j = 0; j < n; ++j) {
        xi[j] = -1;
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

// Regions of the workspace.  Sized per item, so that the size does not depend on which items share an input; a call
// uses the region of the first item that reads an input for all that share it.
struct BlockSpace {
    size_t rs[PEQA_MAX_BLOCK];       // per-channel item, T > 16: row sums of its input
    size_t dys[PEQA_MAX_BLOCK];      // backward, per-channel item j: bf16(dY (s0 + ds)) [T, N]
    size_t crow[PEQA_MAX_BLOCK];     //   its row factors [T]
    size_t partial[PEQA_MAX_BLOCK];  //   per-token-tile partials of its scale gradient [tiles_t, N]
    size_t table[PEQA_MAX_BLOCK];    // group-wise item j: its (s, b) table [G, N, 2]
    size_t xt[PEQA_MAX_BLOCK];       // backward, group-wise item j: step-major transposed copy of its input [K, T']
    size_t dyt[PEQA_MAX_BLOCK];      //   the same of its dY [N, T']
    size_t pc[PEQA_MAX_BLOCK];       //   scale gradient per 64-feature chunk [N, K / 64]
    size_t total;
};

BlockSpace carve_block(int32_t n, const peqa_block_item *items, int32_t T, int32_t op)
{
    BlockSpace w{};
    const size_t tiles_t = ((size_t)T + 127) / 128, Tp = ((size_t)T + 63) / 64 * 64;
    size_t off = 0;
    for (int j = 0; j < n; ++j) {
        const peqa_layout *L = &items[j].layout;
        const size_t N = (size_t)L->n_out, K = (size_t)L->k_in;
        if (grouped(L)) {
            w.table[j] = off; off += round256(N * (size_t)groups(L) * 2 * sizeof(float));
            if (op == PEQA_OP_BWD) {
                w.xt[j] = off;  off += round256(K * Tp * sizeof(uint16_t));
                w.dyt[j] = off; off += round256(N * Tp * sizeof(uint16_t));
                w.pc[j] = off;  off += round256(N * (K / 64) * sizeof(float));
            }
            continue;
        }
        w.rs[j] = off; off += round256((size_t)T * 2 * sizeof(float));
        if (op == PEQA_OP_BWD) {
            w.dys[j] = off;     off += round256((size_t)T * N * sizeof(uint16_t));
            w.crow[j] = off;    off += round256((size_t)T * sizeof(float));
            w.partial[j] = off; off += round256(tiles_t * N * sizeof(float));
        }
    }
    w.total = off ? off : 256;
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
// multiple of 8.  A launch without tiles is made of auxiliary workgroups alone: four per compute unit.
void place_aux(peqa::MultiArgs &m, int aux_wgs)
{
    int total = 0;
    for (int j = 0; j < m.n_jobs; ++j) total += peqa::gemm_multi_wgs(m.job[j].a.tiles_t, m.job[j].a.tiles_c);
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    const int first_round = 2 * cus / 8 * 8;
    m.aux_begin = total < first_round ? total : first_round;
    if (total == 0) aux_wgs = 4 * cus / 8 * 8;
    m.aux_wgs = (m.n_sdy > 0 || m.n_red > 0 || m.n_tp > 0) ? aux_wgs : 0;
}

// The dX tiles of a group-wise layer whose group size is a multiple of 128 scale their activation fragments (the tiles
// of the multi-contraction launches are all of the four-wave form, and block items have integer zero-points).
bool a_side(const peqa_layout *L) { return L->group_size > 0 && L->group_size % 128 == 0; }

// Tables of every group-wise item (of those whose dX is wanted, in the form their dX tiles read, if only_dx): one launch.
peqa_status group_tables(int32_t n, const peqa_block_item *items, uint8_t *ws, const BlockSpace &w, bool only_dx,
                         hipStream_t s)
{
    peqa::GroupTableMulti gt{};
    for (int j = 0; j < n; ++j) {
        const peqa_block_item &it = items[j];
        if (!grouped(&it.layout) || (only_dx && !it.dX)) continue;
        const int i = gt.n++;
        gt.s0[i] = it.s0; gt.ds[i] = it.ds; gt.z0[i] = it.z0;
        gt.sb[i] = reinterpret_cast<float *>(ws + w.table[j]);
        gt.N[i] = it.layout.n_out; gt.G[i] = groups(&it.layout);
        gt.a_side[i] = only_dx && a_side(&it.layout);
    }
    if (gt.n == 0) return PEQA_OK;
    for (int i = gt.n; i < peqa::GT_MAX; ++i) {
        gt.s0[i] = gt.s0[0]; gt.ds[i] = gt.ds[0]; gt.z0[i] = gt.z0[0]; gt.sb[i] = gt.sb[0]; gt.N[i] = gt.N[0]; gt.G[i] = gt.G[0];
        gt.a_side[i] = gt.a_side[0];
    }
    return dev_status(peqa::launch_group_table_multi(gt, s));
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
    const int bits = items[0].layout.bits;
    // row sums of every distinct input of the per-channel items: one launch
    const float *rs[PEQA_MAX_BLOCK] = {nullptr};
    {
        peqa::RowsumMulti r{};
        int nr = 0;
        for (int i = 0; i < nx; ++i) {
            float *dst = nullptr;
            for (int j = 0; j < n; ++j) {
                if (xi[j] != i || grouped(&items[j].layout)) continue;
                if (!dst) dst = reinterpret_cast<float *>(ws + w.rs[j]);
                if (items[j].row_sums) { dst = items[j].row_sums; break; }
            }
            if (!dst) continue;
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
    st = group_tables(n, items, ws, w, false, s);
    if (st != PEQA_OK) return st;
    // all per-channel contractions in one launch, all group-wise ones in another
    peqa::MultiArgs m{}, mg{};
    for (int j = 0; j < n; ++j) {
        const peqa_block_item &it = items[j];
        const int N = it.layout.n_out, K = it.layout.k_in;
        const bool gw = grouped(&it.layout);
        peqa::MultiArgs &dst = gw ? mg : m;
        peqa::MultiJob &job = dst.job[dst.n_jobs++];
        job.mode = peqa::MODE_Y;
        peqa::GemmArgs &a = job.a;
        a.packed = it.packed; a.A = it.X; a.T = T; a.KC = K; a.C = N; a.K = K;
        a.tiles_c = (N + 255) / 256; a.tiles_t = (T + 127) / 128;
        a.out = it.Y;
        if (gw) {
            a.N = N; a.gsz = it.layout.group_size; a.G = groups(&it.layout);
            a.sb = reinterpret_cast<const float *>(ws + w.table[j]);
        } else {
            a.s0 = it.s0; a.ds = it.ds; a.z0 = it.z0; a.rs = rs[xi[j]];
        }
    }
    if (m.n_jobs > 0) {
        sort_jobs(m);
        place_aux(m, 0);
        if (peqa::launch_gemm_multi(bits, false, m, s) != hipSuccess) return PEQA_ERR_DEVICE;
    }
    if (mg.n_jobs > 0) {
        sort_jobs(mg);
        place_aux(mg, 0);
        if (peqa::launch_gemm_multi(bits, true, mg, s) != hipSuccess) return PEQA_ERR_DEVICE;
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
    const int tiles_t = (T + 127) / 128, Tp = (T + 63) / 64 * 64;
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
            float *dst = nullptr;
            for (int j = 0; j < n; ++j)
                if (xi[j] == i && !grouped(&items[j].layout)) {
                    wanted = wanted || items[j].d_ds != nullptr;
                    if (items[j].row_sums) have = items[j].row_sums;
                    if (!dst) dst = reinterpret_cast<float *>(ws + w.rs[j]);
                }
            if (have || !wanted) { rs[i] = have; continue; }
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
        if (peqa::launch_gemm_multi(bits, false, ma, s) != hipSuccess) return PEQA_ERR_DEVICE;
    }
    if (mb.n_jobs > 0 || mb.n_red > 0) {
        sort_jobs(mb);
        place_aux(mb, 64);
        if (peqa::launch_gemm_multi(bits, false, mb, s) != hipSuccess) return PEQA_ERR_DEVICE;
    }

    // ---- group-wise items.  Their (s, b) tables in one launch; every dX contraction in one launch, whose auxiliary
    // workgroups write the transposed copies of X (once per distinct input) and dY that the scale gradients read;
    // the token contractions of all scale gradients in one launch; the sums of their chunks in one launch.
    st = group_tables(n, items, ws, w, true, s);
    if (st != PEQA_OK) return st;
    peqa::MultiArgs mg{}, mg2{};                          // dX jobs that scale their activation fragments; the others
    peqa::DwMultiArgs dw{};
    const uint16_t *xt_of[PEQA_MAX_BLOCK] = {nullptr};
    int tp_tiles = 0;
    for (int j = 0; j < n; ++j) {
        const peqa_block_item &it = items[j];
        if (!grouped(&it.layout)) continue;
        const int N = it.layout.n_out, K = it.layout.k_in, G = groups(&it.layout);
        if (it.dX) {
            peqa::MultiArgs &dst = a_side(&it.layout) ? mg : mg2;
            peqa::MultiJob &job = dst.job[dst.n_jobs++];
            job.mode = peqa::MODE_DX;
            peqa::GemmArgs &a = job.a;
            a.packed = it.packed; a.A = it.dY; a.T = T; a.KC = N; a.C = K; a.K = K;
            a.tiles_c = (K + 255) / 256; a.tiles_t = tiles_t;
            a.N = N; a.gsz = it.layout.group_size; a.G = G; a.a_side = a_side(&it.layout);
            a.sb = reinterpret_cast<const float *>(ws + w.table[j]); a.out = it.dX;
        }
        if (it.d_ds) {
            if (!xt_of[xi[j]]) {
                uint16_t *xt = reinterpret_cast<uint16_t *>(ws + w.xt[j]);
                peqa::TransposeJob &t = mg.tp[mg.n_tp++];
                t.src = it.X; t.dst = xt; t.T = T; t.C = K; t.Tp = Tp;
                tp_tiles += (Tp / 64) * (K / 64);
                t.tile_end = tp_tiles;
                xt_of[xi[j]] = xt;
            }
            uint16_t *dyt = reinterpret_cast<uint16_t *>(ws + w.dyt[j]);
            peqa::TransposeJob &t = mg.tp[mg.n_tp++];
            t.src = it.dY; t.dst = dyt; t.T = T; t.C = N; t.Tp = Tp;
            tp_tiles += (Tp / 64) * (N / 64);
            t.tile_end = tp_tiles;
            peqa::DwArgs &a = dw.job[dw.n_jobs];
            a.Xt = xt_of[xi[j]]; a.dYt = dyt; a.packed = it.packed; a.z0 = it.z0;
            a.pc = reinterpret_cast<float *>(ws + w.pc[j]);
            a.N = N; a.K = K; a.Tp = Tp; a.gsz = it.layout.group_size; a.G = G;
            a.tiles_f = (K + 255) / 256; a.tiles_c = (N + 255) / 256;
            dw.d_ds[dw.n_jobs++] = it.d_ds;
        }
    }
    if (mg.n_jobs > 0 || mg.n_tp > 0) {
        sort_jobs(mg);
        place_aux(mg, 128);
        if (peqa::launch_gemm_multi(bits, true, mg, s) != hipSuccess) return PEQA_ERR_DEVICE;
    }
    if (mg2.n_jobs > 0) {
        sort_jobs(mg2);
        place_aux(mg2, 0);
        if (peqa::launch_gemm_multi(bits, true, mg2, s) != hipSuccess) return PEQA_ERR_DEVICE;
    }
    if (dw.n_jobs > 0) {
        if (peqa::launch_dw_multi(bits, dw, s) != hipSuccess) return PEQA_ERR_DEVICE;
        if (peqa::launch_chunk_reduce_multi(dw, s) != hipSuccess) return PEQA_ERR_DEVICE;
    }
    return PEQA_OK;
}

}  // extern "C"
