// C-ABI of the PEQA library (include/peqa.h): host-side validation, workspace carving and
// kernel sequencing.  No device memory is allocated here and nothing synchronises, except
// the benchmark tracing hooks at the bottom.
#include "../../include/peqa.h"

#include <limits.h>
#include <math.h>
#include <string.h>

#include "peqa_host.h"

using namespace peqa::host;

namespace {

constexpr int PEQA_GEMV_MAX_T = GEMV_MAX_T;

struct Workspace {
    size_t rs, dys, crow, partial, table, rsz, zpartial, xt, dyt, pc, total;
};

Workspace carve(const peqa_layout *L, int32_t T, int32_t op)
{
    if (op == PEQA_OP_FWD_Z && T > PEQA_GEMV_MAX_T) return carve(L, T, PEQA_OP_FWD);
    if (op == PEQA_OP_BWD_Z) {
        // the plain backward's needs, then the group sums of X and the partials of the zero-point gradient
        Workspace w = carve(L, T, PEQA_OP_BWD);
        const size_t slices = ((size_t)T + peqa::KEPT_ROWS - 1) / peqa::KEPT_ROWS;
        const size_t NG = (size_t)L->n_out * (size_t)groups(L);
        w.rsz = w.total;      w.total += round256((size_t)T * groups(L) * sizeof(float));
        w.zpartial = w.total; w.total += round256(slices * NG * sizeof(float));
        return w;
    }
    Workspace w{};
    const size_t N = (size_t)L->n_out, G = (size_t)groups(L);
    const size_t tiles_t = ((size_t)T + 127) / 128;
    size_t off = 0;
    if (op == PEQA_OP_FWD_KEEP || op == PEQA_OP_BWD_KEPT) {
        // per-channel only; the forward always takes the tiled contraction (it writes P from its epilogue)
        if (op == PEQA_OP_FWD_KEEP) {
            w.rs = off;      off += round256((size_t)T * 2 * sizeof(float));
        } else {
            const size_t slices = ((size_t)T + peqa::KEPT_ROWS - 1) / peqa::KEPT_ROWS;
            w.dys = off;     off += round256((size_t)T * N * sizeof(uint16_t));
            w.crow = off;    off += round256((size_t)T * sizeof(float));
            w.partial = off; off += round256(slices * N * sizeof(float));
        }
        w.total = off;
        return w;
    }
    if ((op == PEQA_OP_FWD || op == PEQA_OP_FWD_Z) && T <= PEQA_GEMV_MAX_T) {
        // with a trained zero-point offset a slice of a group-wise layer spans fewer groups: more slices
        const GemvItem one{L, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
        w.partial = off; off += round256(gemv_partial_bytes(1, &one, T, false, op == PEQA_OP_FWD));
        if (off == 0) off = 256;                               // a single slice needs none; 0 would read as "invalid"
        w.total = off;
        return w;
    }
    if (grouped(L)) {
        // group-wise: (s, b) table for the forward / dX contraction; row sums of X over every scale
        // group and per-(token tile, channel, group) partials for the scale gradient
        w.table = off;   off += round256(N * G * 2 * sizeof(float));
        if (op == PEQA_OP_BWD) {
            const size_t Tp = ((size_t)T + 63) / 64 * 64, K = (size_t)L->k_in;
            w.rs = off;      off += round256((size_t)T * G * sizeof(float));
            w.partial = off; off += round256(tiles_t * N * G * sizeof(float));
            // scale gradient by the token contraction: both operands transposed, per-chunk results
            w.xt = off;      off += round256(K * Tp * sizeof(uint16_t));
            w.dyt = off;     off += round256(N * Tp * sizeof(uint16_t));
            w.pc = off;      off += round256(N * (K / 64) * sizeof(float));
        }
        w.total = off;
        return w;
    }
    w.rs = off;      off += round256((size_t)T * 2 * sizeof(float));
    if (op == PEQA_OP_BWD) {
        w.dys = off;     off += round256((size_t)T * N * sizeof(uint16_t));
        w.crow = off;    off += round256((size_t)T * sizeof(float));
        w.partial = off; off += round256(tiles_t * N * G * sizeof(float));
    }
    w.total = off;
    return w;
}

peqa_status fwd_per_channel(const peqa_layout *L, const uint32_t *packed, const float *s0, const float *ds,
                            const uint8_t *z0, const float *dz, const uint16_t *X, int32_t T, uint16_t *Y, float *P,
                            const float *rs, hipStream_t s);

// Scale gradient of group-wise layers: by the contraction over tokens (default), or, with the option
// grouped_dds = 1, by the contraction over features, one pair of scale groups per workgroup: the older,
// slower route, kept for comparison.
bool grouped_dds_by_tokens() { return peqa::options().grouped_dds == 0; }

}  // namespace

extern "C" {

peqa_status peqa_check_layout(const peqa_layout *L)
{
    if (!L) return PEQA_ERR_NULL;
    if (L->bits != 3 && L->bits != 4) return PEQA_ERR_BITS;
    if (L->n_out <= 0 || L->k_in <= 0) return PEQA_ERR_SHAPE;
    if (L->n_out % 128 != 0 || L->k_in % 128 != 0) return PEQA_ERR_SHAPE;
    if ((int64_t)L->n_out * L->k_in > ((int64_t)1 << 40)) return PEQA_ERR_SHAPE;
    if (L->group_size < 0) return PEQA_ERR_GROUP;
    if (L->group_size > 0 && (L->group_size % 64 != 0 || L->k_in % L->group_size != 0)) return PEQA_ERR_GROUP;
    return PEQA_OK;
}

size_t peqa_packed_words(const peqa_layout *L)
{
    if (peqa_check_layout(L) != PEQA_OK) return 0;
    return (size_t)L->n_out * (size_t)L->k_in * (size_t)L->bits / 32u;
}

size_t peqa_num_scales(const peqa_layout *L)
{
    if (peqa_check_layout(L) != PEQA_OK) return 0;
    return (size_t)L->n_out * (size_t)groups(L);
}

size_t peqa_workspace_bytes(const peqa_layout *L, int32_t T, int32_t op)
{
    if (peqa_check_layout(L) != PEQA_OK || T < 1) return 0;
    if (op == PEQA_OP_FWD_KEEP || op == PEQA_OP_BWD_KEPT) {
        if (grouped(L)) return 0;
    } else if (op != PEQA_OP_FWD && op != PEQA_OP_BWD && op != PEQA_OP_FWD_Z && op != PEQA_OP_BWD_Z) {
        return 0;
    }
    return carve(L, T, op).total;
}

peqa_status peqa_set_option(int32_t option, int32_t value)
{
    peqa::Options &o = peqa::options();
    switch (option) {
    case PEQA_OPT_GEMM_WAVES:
        if (value != 0 && value != 4 && value != 8) return PEQA_ERR_PARAM;
        o.gemm_waves = value;
        return PEQA_OK;
    case PEQA_OPT_BWD_PAIR:
        if (value < -1 || value > 1) return PEQA_ERR_PARAM;
        o.bwd_pair = value;
        return PEQA_OK;
    case PEQA_OPT_GROUPED_DDS:
        if (value != 0 && value != 1) return PEQA_ERR_PARAM;
        o.grouped_dds = value;
        return PEQA_OK;
    default:
        return PEQA_ERR_PARAM;
    }
}

int32_t peqa_get_option(int32_t option)
{
    const peqa::Options &o = peqa::options();
    switch (option) {
    case PEQA_OPT_GEMM_WAVES: return o.gemm_waves;
    case PEQA_OPT_BWD_PAIR: return o.bwd_pair;
    case PEQA_OPT_GROUPED_DDS: return o.grouped_dds;
    default: return INT32_MIN;
    }
}

const char *peqa_status_string(int32_t status)
{
    switch (status) {
    case PEQA_OK: return "ok";
    case PEQA_ERR_NULL: return "required pointer is NULL";
    case PEQA_ERR_SHAPE: return "unsupported shape";
    case PEQA_ERR_BITS: return "bits must be 3 or 4";
    case PEQA_ERR_GROUP: return "invalid group size";
    case PEQA_ERR_ALIGN: return "device pointer not 16-byte aligned";
    case PEQA_ERR_WORKSPACE: return "workspace missing or too small";
    case PEQA_ERR_DEVICE: return "HIP runtime error";
    case PEQA_ERR_PARAM: return "invalid scalar parameter";
    default: return "unknown status";
    }
}

peqa_status peqa_bit_location(const peqa_layout *L, int32_t i, int32_t k, int32_t t, size_t *word, int32_t *bit)
{
    peqa_status st = peqa_check_layout(L);
    if (st != PEQA_OK) return st;
    if (!word || !bit) return PEQA_ERR_NULL;
    if (i < 0 || i >= L->n_out || k < 0 || k >= L->k_in || t < 0 || t >= L->bits) return PEQA_ERR_SHAPE;
    const size_t tile = (size_t)(i >> 7) * (size_t)(L->k_in >> 5) + (size_t)(k >> 5);
    const size_t blk = tile * 64 + (size_t)(((i >> 3) & 15) * 4 + ((k >> 3) & 3));
    const int r = i & 7, c = k & 7;
    if (L->bits == 4) {
        *word = blk * 8 + r;
        *bit = 4 * ((c >> 1) + 4 * (c & 1)) + t;
    } else {
        const int u = 4 * (r >> 1) + (c >> 1), par = r & 1, half = c & 1;
        if (u < 15) {
            *word = blk * 6 + 2 * (u / 5) + par;
            *bit = 16 * half + 3 * (u % 5) + t;
        } else {
            *word = blk * 6 + 2 * t + par;
            *bit = 15 + 16 * half;
        }
    }
    return PEQA_OK;
}

peqa_status peqa_quantize(const peqa_layout *L, const float *W0, uint32_t *packed, float *s0, uint8_t *z0,
                          void *stream)
{
    peqa_status st = peqa_check_layout(L);
    if (st != PEQA_OK) return st;
    if (!W0 || !packed || !s0 || !z0) return PEQA_ERR_NULL;
    if (!aligned16(W0) || !aligned16(packed) || !aligned16(s0) || !aligned16(z0)) return PEQA_ERR_ALIGN;
    return dev_status(peqa::launch_quantize(W0, L->n_out, L->k_in, L->bits, L->group_size, packed, s0, z0,
                                            static_cast<hipStream_t>(stream)));
}

static peqa_status fwd_impl(const peqa_layout *L, const uint32_t *packed, const float *s0, const float *ds,
                            const uint8_t *z0, const float *dz, const uint16_t *X, int32_t T, uint16_t *Y,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    peqa_status st = peqa_check_layout(L);
    if (st != PEQA_OK) return st;
    if (!packed || !s0 || !z0 || !X || !Y) return PEQA_ERR_NULL;
    if (T < 1 || T > (1 << 24)) return PEQA_ERR_SHAPE;
    if (!aligned16(packed) || !aligned16(s0) || !aligned16(z0) || !aligned16(X) || !aligned16(Y) ||
        (ds && !aligned16(ds)) || (dz && !aligned16(dz)))
        return PEQA_ERR_ALIGN;
    const Workspace w = carve(L, T, dz ? PEQA_OP_FWD_Z : PEQA_OP_FWD);
    if (!workspace || workspace_bytes < w.total) return PEQA_ERR_WORKSPACE;
    if (!aligned16(workspace)) return PEQA_ERR_ALIGN;

    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    const int N = L->n_out, K = L->k_in, ksplit = split_point(K);
    if (T <= PEQA_GEMV_MAX_T) {
        const GemvItem item{L, packed, s0, ds, z0, dz, X, Y};
        return gemv_forward(1, &item, T, false, reinterpret_cast<float *>(ws + w.partial), s);
    }
    if (grouped(L)) {
        float *sb = reinterpret_cast<float *>(ws + w.table);
        if (peqa::launch_group_table(s0, ds, z0, dz, N, groups(L), false, sb, s) != hipSuccess) return PEQA_ERR_DEVICE;
        peqa::GemmArgs a{};
        a.packed = packed; a.A = X; a.T = T; a.KC = K; a.C = N; a.K = K;
        a.tiles_c = (N + 255) / 256; a.tiles_t = (T + 127) / 128;
        a.N = N; a.gsz = L->group_size; a.G = groups(L); a.sb = sb; a.out = Y;
        return dev_status(peqa::launch_gemm(L->bits, peqa::MODE_Y, a, s));
    }
    float *rs = reinterpret_cast<float *>(ws + w.rs);
    if (peqa::launch_rowsum(X, T, K, ksplit, rs, s) != hipSuccess) return PEQA_ERR_DEVICE;
    return fwd_per_channel(L, packed, s0, ds, z0, dz, X, T, Y, nullptr, rs, s);
}

peqa_status peqa_quantize_search(const peqa_layout *L, const float *W0, int32_t n_ratios, float min_ratio,
                                 uint32_t *packed, float *s0, uint8_t *z0, void *stream)
{
    peqa_status st = peqa_check_layout(L);
    if (st != PEQA_OK) return st;
    if (!W0 || !packed || !s0 || !z0) return PEQA_ERR_NULL;
    if (n_ratios < 1 || n_ratios > 1024 || !(min_ratio > 0.f) || min_ratio > 1.f) return PEQA_ERR_PARAM;
    if (!aligned16(W0) || !aligned16(packed) || !aligned16(s0) || !aligned16(z0)) return PEQA_ERR_ALIGN;
    if (!peqa::quantize_resident_fits(L->k_in, groups(L), true)) return PEQA_ERR_SHAPE;
    // the grid step, in fp32 as the definition has it
    volatile float span = 1.0f - min_ratio;
    volatile float step = n_ratios > 1 ? span / (float)(n_ratios - 1) : 0.0f;
    return dev_status(peqa::launch_quantize_search(W0, L->n_out, L->k_in, L->bits, L->group_size, n_ratios, step,
                                                   packed, s0, z0, static_cast<hipStream_t>(stream)));
}

peqa_status peqa_linear_fwd(const peqa_layout *L, const uint32_t *packed, const float *s0, const float *ds,
                            const uint8_t *z0, const uint16_t *X, int32_t T, uint16_t *Y, void *workspace,
                            size_t workspace_bytes, void *stream)
{
    return fwd_impl(L, packed, s0, ds, z0, nullptr, X, T, Y, workspace, workspace_bytes, stream);
}

// ---- forward without a caller workspace: the scratch is an array in the library's own device image.
// In host code the array's name is only a handle for the runtime's symbol lookup, never an address: every use of
// its memory goes through the pointer that hipGetSymbolAddress returned for the current device.
}  // extern "C"

static __device__ __align__(256) unsigned char scratch[PEQA_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];     // device address of `scratch` on each device, looked up at first use

peqa_status static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PEQA_ERR_DEVICE;
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PEQA_ERR_DEVICE;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return PEQA_OK;
}
}  // namespace

extern "C" {

peqa_status peqa_linear_fwd_static(const peqa_layout *L, const uint32_t *packed, const float *s0, const float *ds,
                                   const uint8_t *z0, const uint16_t *X, int32_t T, uint16_t *Y, void *stream)
{
    peqa_status st = peqa_check_layout(L);
    if (st != PEQA_OK) return st;
    if (T < 1 || T > (1 << 24)) return PEQA_ERR_SHAPE;
    if (carve(L, T, PEQA_OP_FWD).total > (size_t)PEQA_STATIC_SCRATCH_BYTES) return PEQA_ERR_WORKSPACE;
    if (!packed || !s0 || !z0 || !X || !Y) return PEQA_ERR_NULL;    // before the device is touched
    void *ws = nullptr;
    st = static_scratch(&ws);
    if (st != PEQA_OK) return st;
    return fwd_impl(L, packed, s0, ds, z0, nullptr, X, T, Y, ws, (size_t)PEQA_STATIC_SCRATCH_BYTES, stream);
}

peqa_status peqa_linear_fwd_z(const peqa_layout *L, const uint32_t *packed, const float *s0, const float *ds,
                              const uint8_t *z0, const float *dz, const uint16_t *X, int32_t T, uint16_t *Y,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    return fwd_impl(L, packed, s0, ds, z0, dz, X, T, Y, workspace, workspace_bytes, stream);
}

peqa_status peqa_linear_fwd_keep(const peqa_layout *L, const uint32_t *packed, const float *s0, const float *ds,
                                 const uint8_t *z0, const uint16_t *X, int32_t T, uint16_t *Y, float *P,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    peqa_status st = peqa_check_layout(L);
    if (st != PEQA_OK) return st;
    if (grouped(L)) return PEQA_ERR_GROUP;
    if (!packed || !s0 || !z0 || !X || !Y || !P) return PEQA_ERR_NULL;
    if (T < 1 || T > (1 << 24)) return PEQA_ERR_SHAPE;
    if (!aligned16(packed) || !aligned16(s0) || !aligned16(z0) || !aligned16(X) || !aligned16(Y) || !aligned16(P) ||
        (ds && !aligned16(ds)))
        return PEQA_ERR_ALIGN;
    const Workspace w = carve(L, T, PEQA_OP_FWD_KEEP);
    if (!workspace || workspace_bytes < w.total) return PEQA_ERR_WORKSPACE;
    if (!aligned16(workspace)) return PEQA_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *rs = reinterpret_cast<float *>(static_cast<uint8_t *>(workspace) + w.rs);
    if (peqa::launch_rowsum(X, T, L->k_in, split_point(L->k_in), rs, s) != hipSuccess) return PEQA_ERR_DEVICE;
    return fwd_per_channel(L, packed, s0, ds, z0, nullptr, X, T, Y, P, rs, s);
}

}  // extern "C"

namespace {
// Per-channel forward contraction for T > 16, the row sums of X already in `rs`.
peqa_status fwd_per_channel(const peqa_layout *L, const uint32_t *packed, const float *s0, const float *ds,
                            const uint8_t *z0, const float *dz, const uint16_t *X, int32_t T, uint16_t *Y, float *P,
                            const float *rs, hipStream_t s)
{
    const int N = L->n_out, K = L->k_in;
    peqa::GemmArgs a{};
    a.packed = packed; a.A = X; a.T = T; a.KC = K; a.C = N; a.K = K;
    a.tiles_c = (N + 255) / 256; a.tiles_t = (T + 127) / 128;
    a.s0 = s0; a.ds = ds; a.z0 = z0; a.dz = dz; a.rs = rs; a.out = Y; a.P = P;
    return dev_status(peqa::launch_gemm(L->bits, peqa::MODE_Y, a, s));
}
}  // namespace

extern "C" {

// Forward of several layers that read the same X.
static peqa_status check_fused(int32_t n, const peqa_fwd_item *items, int32_t T)
{
    if (!items) return PEQA_ERR_NULL;
    if (n < 1 || n > PEQA_MAX_FUSED) return PEQA_ERR_PARAM;
    if (T < 1 || T > (1 << 24)) return PEQA_ERR_SHAPE;
    for (int j = 0; j < n; ++j) {
        peqa_status st = peqa_check_layout(&items[j].layout);
        if (st != PEQA_OK) return st;
        if (items[j].layout.k_in != items[0].layout.k_in || items[j].layout.bits != items[0].layout.bits ||
            items[j].layout.group_size != items[0].layout.group_size)
            return PEQA_ERR_PARAM;
    }
    return PEQA_OK;
}

size_t peqa_workspace_bytes_fused(int32_t n, const peqa_fwd_item *items, int32_t T)
{
    if (check_fused(n, items, T) != PEQA_OK) return 0;
    if (T <= PEQA_GEMV_MAX_T) {
        GemvItem gi[PEQA_MAX_FUSED];
        for (int j = 0; j < n; ++j) gi[j] = GemvItem{&items[j].layout, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
        const size_t b = round256(gemv_partial_bytes(n, gi, T, false, true));
        return b ? b : 256;
    }
    size_t need = 0;                                       // layer by layer: the largest single need
    for (int j = 0; j < n; ++j) {
        const size_t b = carve(&items[j].layout, T, PEQA_OP_FWD).total;
        need = b > need ? b : need;
    }
    return need;
}

static peqa_status fwd_fused_impl(int32_t n, const peqa_fwd_item *items, const uint16_t *X, const float *row_sums,
                                  int32_t T, void *workspace, size_t workspace_bytes, void *stream)
{
    if (row_sums && !aligned16(row_sums)) return PEQA_ERR_ALIGN;
    peqa_status st = check_fused(n, items, T);
    if (st != PEQA_OK) return st;
    if (!X) return PEQA_ERR_NULL;
    for (int j = 0; j < n; ++j) {
        const peqa_fwd_item &it = items[j];
        if (!it.packed || !it.s0 || !it.z0 || !it.Y) return PEQA_ERR_NULL;
        if (!aligned16(it.packed) || !aligned16(it.s0) || !aligned16(it.z0) || !aligned16(it.Y) ||
            (it.ds && !aligned16(it.ds)))
            return PEQA_ERR_ALIGN;
    }
    if (!aligned16(X)) return PEQA_ERR_ALIGN;
    const size_t need = peqa_workspace_bytes_fused(n, items, T);
    if (!workspace || workspace_bytes < need) return PEQA_ERR_WORKSPACE;
    if (!aligned16(workspace)) return PEQA_ERR_ALIGN;
    if (T <= PEQA_GEMV_MAX_T) {
        GemvItem gi[PEQA_MAX_FUSED];
        for (int j = 0; j < n; ++j)
            gi[j] = GemvItem{&items[j].layout, items[j].packed, items[j].s0, items[j].ds, items[j].z0, nullptr, X, items[j].Y};
        return gemv_forward(n, gi, T, false, static_cast<float *>(workspace), static_cast<hipStream_t>(stream));
    }
    // the tiled contraction runs the layers one by one; per-channel layers share the row sums of X
    if (!grouped(&items[0].layout)) {
        hipStream_t s = static_cast<hipStream_t>(stream);
        const float *rs = row_sums;
        if (!rs) {
            float *own = static_cast<float *>(workspace);  // carve() puts the row sums first
            if (peqa::launch_rowsum(X, T, items[0].layout.k_in, split_point(items[0].layout.k_in), own, s) != hipSuccess)
                return PEQA_ERR_DEVICE;
            rs = own;
        }
        for (int j = 0; j < n; ++j) {
            const peqa_fwd_item &it = items[j];
            st = fwd_per_channel(&it.layout, it.packed, it.s0, it.ds, it.z0, nullptr, X, T, it.Y, nullptr, rs, s);
            if (st != PEQA_OK) return st;
        }
        return PEQA_OK;
    }
    for (int j = 0; j < n; ++j) {
        const peqa_fwd_item &it = items[j];
        st = peqa_linear_fwd(&it.layout, it.packed, it.s0, it.ds, it.z0, X, T, it.Y, workspace, workspace_bytes, stream);
        if (st != PEQA_OK) return st;
    }
    return PEQA_OK;
}

peqa_status peqa_linear_fwd_fused(int32_t n, const peqa_fwd_item *items, const uint16_t *X, int32_t T,
                                  void *workspace, size_t workspace_bytes, void *stream)
{
    return fwd_fused_impl(n, items, X, nullptr, T, workspace, workspace_bytes, stream);
}

peqa_status peqa_linear_fwd_fused_rs(int32_t n, const peqa_fwd_item *items, const uint16_t *X, const float *row_sums,
                                     int32_t T, void *workspace, size_t workspace_bytes, void *stream)
{
    return fwd_fused_impl(n, items, X, row_sums, T, workspace, workspace_bytes, stream);
}

// Backward shared by peqa_linear_bwd (dz = d_dz = NULL, op = PEQA_OP_BWD) and peqa_linear_bwd_z.
static peqa_status bwd_impl(const peqa_layout *L, const uint32_t *packed, const float *s0, const float *ds,
                            const uint8_t *z0, const float *dz, const uint16_t *X, const float *row_sums,
                            const uint16_t *dY, int32_t T, uint16_t *dX, float *d_ds, float *d_dz, int32_t op,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    if (row_sums && !aligned16(row_sums)) return PEQA_ERR_ALIGN;
    peqa_status st = peqa_check_layout(L);
    if (st != PEQA_OK) return st;
    if (!packed || !s0 || !z0 || !dY) return PEQA_ERR_NULL;
    if ((d_ds || d_dz) && !X) return PEQA_ERR_NULL;
    if (T < 1 || T > (1 << 24)) return PEQA_ERR_SHAPE;
    if (!aligned16(packed) || !aligned16(s0) || !aligned16(z0) || !aligned16(dY) || (X && !aligned16(X)) ||
        (ds && !aligned16(ds)) || (dX && !aligned16(dX)) || (d_ds && !aligned16(d_ds)) || (dz && !aligned16(dz)) ||
        (d_dz && !aligned16(d_dz)))
        return PEQA_ERR_ALIGN;
    const Workspace w = carve(L, T, op);
    if (!workspace || workspace_bytes < w.total) return PEQA_ERR_WORKSPACE;
    if (!aligned16(workspace)) return PEQA_ERR_ALIGN;

    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    const int N = L->n_out, K = L->k_in;
    const int tiles_t = (T + 127) / 128;

    const int slices = (T + peqa::KEPT_ROWS - 1) / peqa::KEPT_ROWS;
    if (grouped(L)) {
        const int G = groups(L);
        float *rsb = reinterpret_cast<float *>(ws + w.rs);
        const bool by_tokens = grouped_dds_by_tokens();
        if ((d_ds && !by_tokens) || d_dz) {
            if (peqa::launch_rowsum_groups(X, T, K, L->group_size, rsb, s) != hipSuccess) return PEQA_ERR_DEVICE;
        }
        if (d_dz) {
            float *zp = reinterpret_cast<float *>(ws + w.zpartial);
            if (peqa::launch_dz_partial(dY, rsb, T, N, G, zp, s) != hipSuccess) return PEQA_ERR_DEVICE;
            if (peqa::launch_dz_finish(zp, slices, (size_t)N * G, s0, ds, d_dz, s) != hipSuccess) return PEQA_ERR_DEVICE;
        }
        const int Tp = (T + 63) / 64 * 64;
        uint16_t *xt = reinterpret_cast<uint16_t *>(ws + w.xt), *dyt = reinterpret_cast<uint16_t *>(ws + w.dyt);
        // When dX is wanted too and its contraction runs two workgroups per compute unit, it goes first and spare
        // workgroups of its launch write the transposed copies that the token contraction needs.
        const bool tp_in_dx = d_ds && by_tokens && dX && peqa::gemm_four_waves(tiles_t * ((K + 255) / 256));
        auto run_dx = [&](bool with_transposes) -> peqa_status {
            float *sb = reinterpret_cast<float *>(ws + w.table);
            // four-wave tiles of a group size that is a multiple of 128, integer zero-points: the scale goes on the
            // activation side
            const bool a_side = L->group_size % 128 == 0 && !dz && peqa::gemm_four_waves(tiles_t * ((K + 255) / 256));
            if (peqa::launch_group_table(s0, ds, z0, dz, N, G, a_side, sb, s) != hipSuccess) return PEQA_ERR_DEVICE;
            peqa::GemmArgs a{};
            a.packed = packed; a.A = dY; a.T = T; a.KC = N; a.C = K; a.K = K;
            a.tiles_c = (K + 255) / 256; a.tiles_t = tiles_t;
            a.N = N; a.gsz = L->group_size; a.G = G; a.sb = sb; a.out = dX; a.a_side = a_side;
            if (with_transposes) {
                a.tp_blocks = (Tp / 64) * (K / 64 + N / 64); a.tp_Tp = Tp; a.tp_X = X; a.tp_Xt = xt; a.tp_dYt = dyt;
            }
            return peqa::launch_gemm(L->bits, peqa::MODE_DX, a, s) == hipSuccess ? PEQA_OK : PEQA_ERR_DEVICE;
        };
        if (tp_in_dx) {
            const peqa_status st = run_dx(true);
            if (st != PEQA_OK) return st;
        }
        if (d_ds && by_tokens) {
            float *pc = reinterpret_cast<float *>(ws + w.pc);
            if (!tp_in_dx) {
                if (peqa::launch_transpose_pad(X, T, K, Tp, xt, s) != hipSuccess) return PEQA_ERR_DEVICE;
                if (peqa::launch_transpose_pad(dY, T, N, Tp, dyt, s) != hipSuccess) return PEQA_ERR_DEVICE;
            }
            peqa::DwArgs a{};
            a.Xt = xt; a.dYt = dyt; a.packed = packed; a.z0 = z0; a.dz = dz; a.pc = pc;
            a.N = N; a.K = K; a.Tp = Tp; a.gsz = L->group_size; a.G = G;
            a.tiles_f = (K + 255) / 256; a.tiles_c = (N + 255) / 256;
            if (peqa::launch_dw(L->bits, a, s) != hipSuccess) return PEQA_ERR_DEVICE;
            if (peqa::launch_chunk_reduce(pc, (size_t)N * G, L->group_size / 64, d_ds, s) != hipSuccess)
                return PEQA_ERR_DEVICE;
        } else if (d_ds) {
            float *partial = reinterpret_cast<float *>(ws + w.partial);
            peqa::GemmArgs a{};
            a.packed = packed; a.A = X; a.T = T; a.KC = K; a.C = N; a.K = K;
            a.tiles_c = (N + 255) / 256; a.tiles_t = tiles_t;
            a.N = N; a.gsz = L->group_size; a.G = G;
            a.z0 = z0; a.dz = dz; a.rs = rsb; a.dY = dY; a.partial = partial;
            if (peqa::launch_gemm(L->bits, peqa::MODE_DDS, a, s) != hipSuccess) return PEQA_ERR_DEVICE;
            if (peqa::launch_reduce_partials(partial, tiles_t, (size_t)N * G, d_ds, s) != hipSuccess)
                return PEQA_ERR_DEVICE;
        }
        if (dX && !tp_in_dx) {
            const peqa_status st = run_dx(false);
            if (st != PEQA_OK) return st;
        }
        return PEQA_OK;
    }

    // The two gradients are independent.  Everything stays in order on the caller's stream: running the two
    // chains, or only their small kernels, beside each other on a second stream measured 2-6 % slower on the 7B
    // block, launched one by one (the events cost more than they hide) and as a captured graph alike.
    // With both gradients wanted, the two contractions go out as one launch of four-wave workgroups, after the
    // scaling of dY and before the sum of the partials (option bwd_pair = 0, or gemm_waves = 8: as launches of
    // their own).  Measured against separate launches: +1 to 2 % on the 7B block at T = 2048, where
    // half the launches have one tile per compute unit and would run in the eight-wave form, +0.2 to 0.9 % on the
    // 13B and 65B blocks; 8 to 18 % less time per backward at T = 16 to 1024 on 4096 x 4096 and 4096 x 11008
    // layers, where each contraction alone fills a fraction of the machine.
    bool pair = d_ds && dX && peqa::gemm_four_waves(1 << 30);
    if (peqa::options().bwd_pair >= 0) pair = d_ds && dX && peqa::options().bwd_pair == 1;
    peqa::GemmArgs a_dds{}, a_dx{};
    if (d_ds) {
        // row sums of X over the two contraction halves: the caller's (peqa_row_sums), or taken here
        const float *rs = row_sums;
        if (!rs) {
            float *own = reinterpret_cast<float *>(ws + w.rs);
            if (peqa::launch_rowsum(X, T, K, split_point(K), own, s) != hipSuccess) return PEQA_ERR_DEVICE;
            rs = own;
        }
        peqa::GemmArgs &a = a_dds;
        a.packed = packed; a.A = X; a.T = T; a.KC = K; a.C = N; a.K = K;
        a.tiles_c = (N + 255) / 256; a.tiles_t = tiles_t;
        a.z0 = z0; a.dz = dz; a.rs = rs; a.dY = dY; a.partial = reinterpret_cast<float *>(ws + w.partial);
    }
    if (dX) {
        peqa::GemmArgs &a = a_dx;
        a.packed = packed; a.A = reinterpret_cast<uint16_t *>(ws + w.dys); a.T = T; a.KC = N; a.C = K; a.K = K;
        a.tiles_c = (K + 255) / 256; a.tiles_t = tiles_t;
        a.crow = reinterpret_cast<float *>(ws + w.crow); a.out = dX;
    }
    float *partial = reinterpret_cast<float *>(ws + w.partial);
    uint16_t *dys = reinterpret_cast<uint16_t *>(ws + w.dys);
    float *crow = reinterpret_cast<float *>(ws + w.crow);
    if (pair) {
        if (peqa::launch_scale_dy(dY, s0, ds, z0, dz, T, N, dys, crow, nullptr, 0, 0, nullptr, s) != hipSuccess)
            return PEQA_ERR_DEVICE;
        if (peqa::launch_gemm_bwd_pair(L->bits, a_dds, a_dx, s) != hipSuccess) return PEQA_ERR_DEVICE;
        if (peqa::launch_reduce_partials(partial, tiles_t, (size_t)N, d_ds, s) != hipSuccess) return PEQA_ERR_DEVICE;
    } else {
        // one after the other; when dX follows the scale gradient, the sum of its partials rides in the launch
        // that scales dY
        if (d_ds) {
            if (peqa::launch_gemm(L->bits, peqa::MODE_DDS, a_dds, s) != hipSuccess) return PEQA_ERR_DEVICE;
            if (!dX && peqa::launch_reduce_partials(partial, tiles_t, (size_t)N, d_ds, s) != hipSuccess)
                return PEQA_ERR_DEVICE;
        }
        if (dX) {
            if (peqa::launch_scale_dy(dY, s0, ds, z0, dz, T, N, dys, crow, partial, tiles_t, d_ds ? (size_t)N : 0, d_ds,
                                      s) != hipSuccess)
                return PEQA_ERR_DEVICE;
            if (peqa::launch_gemm(L->bits, peqa::MODE_DX, a_dx, s) != hipSuccess) return PEQA_ERR_DEVICE;
        }
    }
    if (d_dz) {
        // sums of every row of X (one group spanning K), then the two-stage column reduction
        float *rsz = reinterpret_cast<float *>(ws + w.rsz);
        float *zp = reinterpret_cast<float *>(ws + w.zpartial);
        if (peqa::launch_rowsum_groups(X, T, K, K, rsz, s) != hipSuccess) return PEQA_ERR_DEVICE;
        if (peqa::launch_dz_partial(dY, rsz, T, N, 1, zp, s) != hipSuccess) return PEQA_ERR_DEVICE;
        if (peqa::launch_dz_finish(zp, slices, (size_t)N, s0, ds, d_dz, s) != hipSuccess) return PEQA_ERR_DEVICE;
    }
    return PEQA_OK;
}

peqa_status peqa_linear_bwd(const peqa_layout *L, const uint32_t *packed, const float *s0, const float *ds,
                            const uint8_t *z0, const uint16_t *X, const uint16_t *dY, int32_t T, uint16_t *dX,
                            float *d_ds, void *workspace, size_t workspace_bytes, void *stream)
{
    return bwd_impl(L, packed, s0, ds, z0, nullptr, X, nullptr, dY, T, dX, d_ds, nullptr, PEQA_OP_BWD, workspace,
                    workspace_bytes, stream);
}

peqa_status peqa_row_sums(const uint16_t *X, int32_t T, int32_t K, float *row_sums, void *stream)
{
    if (!X || !row_sums) return PEQA_ERR_NULL;
    if (T < 1 || T > (1 << 24) || K < 128 || K % 128 != 0) return PEQA_ERR_SHAPE;
    if (!aligned16(X) || !aligned16(row_sums)) return PEQA_ERR_ALIGN;
    return dev_status(peqa::launch_rowsum(X, T, K, split_point(K), row_sums, static_cast<hipStream_t>(stream)));
}

peqa_status peqa_linear_bwd_rs(const peqa_layout *L, const uint32_t *packed, const float *s0, const float *ds,
                               const uint8_t *z0, const uint16_t *X, const float *row_sums, const uint16_t *dY,
                               int32_t T, uint16_t *dX, float *d_ds, void *workspace, size_t workspace_bytes,
                               void *stream)
{
    return bwd_impl(L, packed, s0, ds, z0, nullptr, X, row_sums, dY, T, dX, d_ds, nullptr, PEQA_OP_BWD, workspace,
                    workspace_bytes, stream);
}

peqa_status peqa_linear_bwd_z(const peqa_layout *L, const uint32_t *packed, const float *s0, const float *ds,
                              const uint8_t *z0, const float *dz, const uint16_t *X, const uint16_t *dY, int32_t T,
                              uint16_t *dX, float *d_ds, float *d_dz, void *workspace, size_t workspace_bytes,
                              void *stream)
{
    return bwd_impl(L, packed, s0, ds, z0, dz, X, nullptr, dY, T, dX, d_ds, d_dz, PEQA_OP_BWD_Z, workspace,
                    workspace_bytes, stream);
}

peqa_status peqa_linear_bwd_kept(const peqa_layout *L, const uint32_t *packed, const float *s0, const float *ds,
                                 const uint8_t *z0, const float *P, const uint16_t *dY, int32_t T, uint16_t *dX,
                                 float *d_ds, void *workspace, size_t workspace_bytes, void *stream)
{
    peqa_status st = peqa_check_layout(L);
    if (st != PEQA_OK) return st;
    if (grouped(L)) return PEQA_ERR_GROUP;
    if (!packed || !s0 || !z0 || !dY) return PEQA_ERR_NULL;
    if (d_ds && !P) return PEQA_ERR_NULL;
    if (T < 1 || T > (1 << 24)) return PEQA_ERR_SHAPE;
    if (!aligned16(packed) || !aligned16(s0) || !aligned16(z0) || !aligned16(dY) || (P && !aligned16(P)) ||
        (ds && !aligned16(ds)) || (dX && !aligned16(dX)) || (d_ds && !aligned16(d_ds)))
        return PEQA_ERR_ALIGN;
    const Workspace w = carve(L, T, PEQA_OP_BWD_KEPT);
    if (!workspace || workspace_bytes < w.total) return PEQA_ERR_WORKSPACE;
    if (!aligned16(workspace)) return PEQA_ERR_ALIGN;

    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    const int N = L->n_out, K = L->k_in;
    if (d_ds) {
        float *partial = reinterpret_cast<float *>(ws + w.partial);
        const int slices = (T + peqa::KEPT_ROWS - 1) / peqa::KEPT_ROWS;
        if (peqa::launch_dds_kept(dY, P, T, N, partial, s) != hipSuccess) return PEQA_ERR_DEVICE;
        if (!dX && peqa::launch_reduce_partials(partial, slices, (size_t)N, d_ds, s) != hipSuccess) return PEQA_ERR_DEVICE;
    }
    if (dX) {
        uint16_t *dys = reinterpret_cast<uint16_t *>(ws + w.dys);
        float *crow = reinterpret_cast<float *>(ws + w.crow);
        const int slices = (T + peqa::KEPT_ROWS - 1) / peqa::KEPT_ROWS;
        if (peqa::launch_scale_dy(dY, s0, ds, z0, nullptr, T, N, dys, crow, reinterpret_cast<const float *>(ws + w.partial),
                                  slices, d_ds ? (size_t)N : 0, d_ds, s) != hipSuccess)
            return PEQA_ERR_DEVICE;
        peqa::GemmArgs a{};
        a.packed = packed; a.A = dys; a.T = T; a.KC = N; a.C = K; a.K = K;
        a.tiles_c = (K + 255) / 256; a.tiles_t = (T + 127) / 128;
        a.crow = crow; a.out = dX;
        if (peqa::launch_gemm(L->bits, peqa::MODE_DX, a, s) != hipSuccess) return PEQA_ERR_DEVICE;
    }
    return PEQA_OK;
}

peqa_status peqa_scale_update(size_t n_scales, float *ds, const float *d_ds, float *m, float *v, const float *s0,
                              const peqa_adamw *opt, void *stream)
{
    if (!ds || !d_ds || !m || !v || !s0 || !opt) return PEQA_ERR_NULL;
    if (n_scales == 0 || n_scales > ((size_t)1 << 38)) return PEQA_ERR_SHAPE;
    if (opt->step < 1 || !(opt->beta1 >= 0.f && opt->beta1 < 1.f) || !(opt->beta2 >= 0.f && opt->beta2 < 1.f) ||
        !(opt->eps >= 0.f) || !(opt->lr == opt->lr) || !(opt->weight_decay == opt->weight_decay))
        return PEQA_ERR_PARAM;
    if (!aligned16(ds) || !aligned16(d_ds) || !aligned16(m) || !aligned16(v) || !aligned16(s0)) return PEQA_ERR_ALIGN;
    const double c1 = 1.0 - pow((double)opt->beta1, (double)opt->step);
    const double c2 = 1.0 - pow((double)opt->beta2, (double)opt->step);
    return dev_status(peqa::launch_adamw(n_scales, ds, d_ds, m, v, s0, opt->lr, opt->beta1, opt->beta2, opt->eps,
                                         opt->weight_decay, (float)(1.0 / c1), (float)(1.0 / c2),
                                         static_cast<hipStream_t>(stream)));
}

peqa_status peqa_device_info(int32_t *compute_units, int32_t *clock_khz)
{
    if (!compute_units || !clock_khz) return PEQA_ERR_NULL;
    int dev = 0, cus = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev) != hipSuccess)
        return PEQA_ERR_DEVICE;
    *compute_units = cus;
    *clock_khz = khz;
    return PEQA_OK;
}

peqa_status peqa_scale_update_multi(int32_t n, const peqa_update_item *items, const peqa_adamw *opt, void *stream)
{
    if (!items || !opt) return PEQA_ERR_NULL;
    if (n < 1 || n > PEQA_MAX_UPDATE) return PEQA_ERR_PARAM;
    if (opt->step < 1 || !(opt->beta1 >= 0.f && opt->beta1 < 1.f) || !(opt->beta2 >= 0.f && opt->beta2 < 1.f) ||
        !(opt->eps >= 0.f) || !(opt->lr == opt->lr) || !(opt->weight_decay == opt->weight_decay))
        return PEQA_ERR_PARAM;
    peqa::AdamwMulti a{};
    unsigned long long total = 0;
    for (int j = 0; j < n; ++j) {
        const peqa_update_item &it = items[j];
        if (!it.ds || !it.d_ds || !it.m || !it.v || !it.s0) return PEQA_ERR_NULL;
        if (it.n_scales == 0 || it.n_scales > ((size_t)1 << 38)) return PEQA_ERR_SHAPE;
        if (!aligned16(it.ds) || !aligned16(it.d_ds) || !aligned16(it.m) || !aligned16(it.v) || !aligned16(it.s0))
            return PEQA_ERR_ALIGN;
        total += it.n_scales;
        a.ds[j] = it.ds; a.g[j] = it.d_ds; a.m[j] = it.m; a.v[j] = it.v; a.s0[j] = it.s0; a.end[j] = total;
    }
    if (total > ((unsigned long long)1 << 38)) return PEQA_ERR_SHAPE;
    for (int j = n; j < peqa::ADAMW_MAX_TENSORS; ++j) {
        a.ds[j] = a.ds[n - 1]; a.g[j] = a.g[n - 1]; a.m[j] = a.m[n - 1]; a.v[j] = a.v[n - 1]; a.s0[j] = a.s0[n - 1];
        a.end[j] = total;
    }
    a.n_tensors = n;
    const double c1 = 1.0 - pow((double)opt->beta1, (double)opt->step);
    const double c2 = 1.0 - pow((double)opt->beta2, (double)opt->step);
    return dev_status(peqa::launch_adamw_multi(a, opt->lr, opt->beta1, opt->beta2, opt->eps, opt->weight_decay,
                                               (float)(1.0 / c1), (float)(1.0 / c2), static_cast<hipStream_t>(stream)));
}

}  // extern "C"

// ---------------------------------------------------------------------------------------
// Benchmark tracing: HIP events around every launch while enabled.
// ---------------------------------------------------------------------------------------
namespace peqa {
namespace host {

void gemv_slicing(int n, const GemvItem *items, int32_t T, bool block_plan, bool zbyte, int *S)
{
    if (block_plan) {
        int N[GEMV_MAX_LAYERS], K[GEMV_MAX_LAYERS], chunk[GEMV_MAX_LAYERS];
        for (int j = 0; j < n; ++j) {
            N[j] = items[j].L->n_out;
            K[j] = items[j].L->k_in;
            chunk[j] = items[j].L->group_size > 0 ? items[j].L->group_size : items[j].L->k_in;
        }
        gemv_plan(n, N, K, chunk, items[0].L->bits, T, zbyte, S);
        return;
    }
    const peqa_layout *L = items[0].L;
    int n_total = 0;
    for (int j = 0; j < n; ++j) n_total += items[j].L->n_out;
    const int s = gemv_slices(n_total, L->k_in, T, L->group_size > 0 ? L->group_size : L->k_in, zbyte);
    for (int j = 0; j < n; ++j) S[j] = s;
}

size_t gemv_partial_bytes(int n, const GemvItem *items, int32_t T, bool block_plan, bool zbyte)
{
    int S[GEMV_MAX_LAYERS];
    gemv_slicing(n, items, T, block_plan, zbyte, S);
    size_t bytes = 0;
    for (int j = 0; j < n; ++j)
        if (S[j] > 1) bytes += (size_t)S[j] * (size_t)T * (size_t)items[j].L->n_out * sizeof(float);
    return bytes;
}

peqa_status gemv_forward(int n, const GemvItem *items, int32_t T, bool block_plan, float *partial, hipStream_t s)
{
    int S[GEMV_MAX_LAYERS];
    bool zbyte = true;                                         // the kernel takes the same decision from the same pointers
    for (int j = 0; j < n; ++j) zbyte = zbyte && items[j].dz == nullptr;
    gemv_slicing(n, items, T, block_plan, zbyte, S);
    GemvArgs g{};
    int wgs = 0;
    size_t poff = 0;                                           // in floats
    for (int j = 0; j < GEMV_MAX_LAYERS; ++j) {
        if (j < n) {
            const peqa_layout *L = items[j].L;
            if ((uint64_t)T * (uint64_t)L->n_out >= ((uint64_t)1 << 31)) return PEQA_ERR_SHAPE;   // 32-bit indexing in there
            GemvLayer &l = g.layer[j];
            l.packed = items[j].packed; l.s0 = items[j].s0; l.ds = items[j].ds; l.z0 = items[j].z0; l.dz = items[j].dz;
            l.X = items[j].X; l.Y = items[j].Y;
            l.N = L->n_out; l.K = L->k_in; l.G = groups(L);
            l.chunk = L->group_size > 0 ? L->group_size : L->k_in;
            l.S = S[j];
            l.partial = partial + poff;
            if (S[j] > 1) poff += (size_t)S[j] * (size_t)T * (size_t)L->n_out;
            wgs += (L->n_out / 128) * S[j];
            l.wg_end = wgs;
        } else {
            g.layer[j] = g.layer[n - 1];                       // never selected: its wg_end is the total
        }
    }
    g.n_layers = n;
    g.T = T;
    return dev_status(launch_gemv(items[0].L->bits, g, s));
}

}  // namespace host

Options &options()
{
    static Options o;
    return o;
}
}  // namespace peqa

namespace {

struct TraceState {
    bool on = false;
    int cap = 0, used = 0;
    hipEvent_t *ev = nullptr;     // 2 per launch
    int *kid = nullptr;
} g_trace;
char g_trace_prefix[32] = "";     // only kernels whose name starts with this are bracketed ("" = all)

const char *const kKernelNames[peqa::KID_COUNT] = {
    "quantize", "rowsum", "gemm_y", "gemm_dds", "gemm_dx", "scale_dy", "reduce_partials", "adamw", "gemv",
    "gemv_finish", "group_table", "dds_kept", "dz_partial", "dz_finish", "transpose_pad", "gemm_dw", "gemm_bwd", "gemm_multi_y", "gemm_multi_dds", "gemm_multi_dx"};

}  // namespace
namespace {

void trace_release()
{
    for (int i = 0; i < 2 * g_trace.cap; ++i) (void)hipEventDestroy(g_trace.ev[i]);
    delete[] g_trace.ev;
    delete[] g_trace.kid;
    g_trace = TraceState{};
}

}  // namespace

namespace peqa {

static bool trace_selected(int kernel_id)
{
    return g_trace_prefix[0] == 0 || strncmp(kKernelNames[kernel_id], g_trace_prefix, strlen(g_trace_prefix)) == 0;
}

void trace_before(int kernel_id, hipStream_t stream)
{
    if (!g_trace.on || g_trace.used >= g_trace.cap || !trace_selected(kernel_id)) return;
    g_trace.kid[g_trace.used] = kernel_id;
    (void)hipEventRecord(g_trace.ev[2 * g_trace.used], stream);
}

void trace_after(int kernel_id, hipStream_t stream)
{
    if (!g_trace.on || g_trace.used >= g_trace.cap || !trace_selected(kernel_id)) return;
    (void)hipEventRecord(g_trace.ev[2 * g_trace.used + 1], stream);
    ++g_trace.used;
}

}  // namespace peqa

extern "C" {

peqa_status peqa_trace_select(const char *prefix)
{
    if (prefix && strlen(prefix) >= sizeof(g_trace_prefix)) return PEQA_ERR_PARAM;
    strncpy(g_trace_prefix, prefix ? prefix : "", sizeof(g_trace_prefix) - 1);
    g_trace_prefix[sizeof(g_trace_prefix) - 1] = 0;
    return PEQA_OK;
}

peqa_status peqa_trace_begin(int32_t max_launches)
{
    if (max_launches < 1 || max_launches > (1 << 20)) return PEQA_ERR_PARAM;
    if (g_trace.ev) trace_release();
    g_trace.ev = new hipEvent_t[2 * (size_t)max_launches];
    g_trace.kid = new int[max_launches];
    g_trace.cap = 0;
    for (int i = 0; i < 2 * max_launches; ++i) {
        if (hipEventCreate(&g_trace.ev[i]) != hipSuccess) {
            g_trace.cap = i / 2;
            trace_release();
            return PEQA_ERR_DEVICE;
        }
    }
    g_trace.cap = max_launches;
    g_trace.used = 0;
    g_trace.on = true;
    return PEQA_OK;
}

int32_t peqa_trace_end(int32_t max_kernels, const char **names, int32_t *launches, float *total_ms)
{
    if (!g_trace.ev) return 0;
    g_trace.on = false;
    int cnt[peqa::KID_COUNT] = {0};
    float ms[peqa::KID_COUNT] = {0.f};
    for (int i = 0; i < g_trace.used; ++i) {
        float t = 0.f;
        if (hipEventSynchronize(g_trace.ev[2 * i + 1]) == hipSuccess &&
            hipEventElapsedTime(&t, g_trace.ev[2 * i], g_trace.ev[2 * i + 1]) == hipSuccess) {
            cnt[g_trace.kid[i]] += 1;
            ms[g_trace.kid[i]] += t;
        }
    }
    int out = 0;
    for (int k = 0; k < peqa::KID_COUNT && out < max_kernels; ++k) {
        if (cnt[k] == 0) continue;
        if (names) names[out] = kKernelNames[k];
        if (launches) launches[out] = cnt[k];
        if (total_ms) total_ms[out] = ms[k];
        ++out;
    }
    trace_release();
    return out;
}

}  // extern "C"
