// C ABI of the CCE- library: argument checks, workspace layout, dispatch.  See include/cce_neg.h for the contract.
#include <hip/hip_runtime.h>
#include <math.h>

#include <string.h>
#include <mutex>
#include <vector>

#include "cce_device.hpp"
#include "cce_kernels.hpp"
#include "cce_tile_shared.hpp"

namespace cce {
namespace {

constexpr size_t kHeaderBytes = 256;  // status word, compaction counters; keeps what follows 256-byte aligned
constexpr int kMaxScratchDevices = 64;

size_t align256(size_t n) { return (n + 255) & ~size_t(255); }

// The matrix-core path runs bf16 shared-negative and full-catalogue descriptors with a supported hidden size.
bool tile_eligible(const cce_desc *d)
{
    if (d->in_dtype != CCE_BF16 || d->neg_mode == CCE_NEG_PER_POSITION || !tile_supports_d(d->d)) return false;
    const int64_t n_cols = (d->neg_mode == CCE_NEG_FULL) ? d->V : d->K;
    return n_cols >= 1;
}
bool use_tile(const cce_desc *d) { return d->algo != CCE_ALGO_GATHER && tile_eligible(d); }
// The forward call forms the hidden-state gradient as well (fuse_dH), where the matrix-core path runs.
bool fused_dH(const cce_desc *d) { return d->fuse_dH != 0 && use_tile(d); }

// Workspace layout of the matrix-core path.  Split factors depend on the descriptor only, so that the size query and
// the launches agree.
struct Layout {
    size_t idx, cnt, coef, de_const, part_m, part_s, part_dH, U, total;
    int splits_x;   // dH pass: candidate range split over at most this many blocks per position block
    int splits_fwd; // forward pass: the same, with its own (cheaper) bound
    int splits_de;  // dE pass: position range split
};

Layout make_layout(const cce_desc *d)
{
    Layout L{};
    const int64_t N = d->N;
    const int64_t n_cols = (d->neg_mode == CCE_NEG_FULL) ? d->V : d->K;
    const int by = 8192 / d->d;  // streamed rows per tile, as in the kernels
    // Upper bounds of the split factors (the launcher picks the factor that fills the chip best, up to these).
    // Splitting only pays when there are few blocks of stationary rows, which bounds splits * rows, hence the
    // partial buffers, by a constant.
    const int64_t xblocks = (N + 127) / 128;
    int sx = (xblocks > 0 && xblocks <= 320) ? (int)(2048 / xblocks) : 1;  // the launcher never splits above 320 blocks
    const int64_t col_tiles = (n_cols + by - 1) / by;
    if (sx > 16) sx = 16;
    if (sx > col_tiles / 2) sx = (int)(col_tiles / 2);
    if (sx < 1) sx = 1;
    L.splits_x = sx;
    // The forward partials are two floats per position and split, so the forward pass may always split: with many
    // blocks it does so only to even out the last round (the launcher decides).
    int sf = (int)(col_tiles / 4);
    if (sf > 8) sf = 8;
    if (sf < sx) sf = sx;
    if (sf < 1) sf = 1;
    L.splits_fwd = sf;
    const int64_t cblocks = (n_cols + 127) / 128;
    int sd = (cblocks > 0) ? (int)(2048 / cblocks) : 1;
    const int64_t pos_tiles = (N + by - 1) / by;
    if (sd > 128) sd = 128;
    if (sd < 8) sd = 8;  // merged by atomics, no buffer depends on it: room to even out a grid of one or two rounds
    if (sd > pos_tiles / 2) sd = (int)(pos_tiles / 2);
    if (sd < 1) sd = 1;
    L.splits_de = sd;

    size_t off = kHeaderBytes;
    L.idx = off;      off += align256((size_t)N * 4);
    L.cnt = off;      off += align256((size_t)N * 4);
    L.coef = off;     off += align256((size_t)N * 4);
    L.de_const = off; off += align256((size_t)N * 8);
    {
        // partial (max, sum) per position and split; the fused forward pass also files them for the rows of its
        // last-round split (at most kTailRows of them)
        size_t words = (sf > 1) ? (size_t)sf * N : 0;
        if (fused_dH(d) && tile_tail_partial_bytes(N, d->d) > 0 && words < (size_t)kTailRows) words = (size_t)kTailRows;
        L.part_m = off;   off += align256(words * 4);
        L.part_s = off;   off += align256(words * 4);
    }
    {
        const size_t split_bytes = (sx > 1) ? (size_t)sx * N * d->d * 4 : 0, tail_bytes = tile_tail_partial_bytes(N, d->d);
        L.part_dH = off;
        off += align256(split_bytes > tail_bytes ? split_bytes : tail_bytes);
    }
    L.U = off;
    if (fused_dH(d)) off += align256((size_t)N * d->d * 4);
    L.total = off;
    return L;
}

__global__ void fill_zero_kernel(int32_t *dst, size_t words)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < words) dst[i] = 0;
}

cce_status check_desc(const cce_desc *d)
{
    if (!d) return CCE_ERR_NULL;
    if (d->N < 0 || d->V <= 0 || d->V > 0x7fffffffLL || d->N > 0x7fffffffLL) return CCE_ERR_SHAPE;
    if (d->d < 8 || d->d > 512 || (d->d % 8) != 0) return CCE_ERR_SHAPE;
    if (d->neg_mode != CCE_NEG_SHARED && d->neg_mode != CCE_NEG_PER_POSITION && d->neg_mode != CCE_NEG_FULL)
        return CCE_ERR_SHAPE;
    if (d->neg_mode != CCE_NEG_FULL && d->K < 0) return CCE_ERR_SHAPE;
    if (d->in_dtype != CCE_F32 && d->in_dtype != CCE_BF16) return CCE_ERR_DTYPE;
    if (d->dH_dtype != CCE_F32 && d->dH_dtype != CCE_BF16) return CCE_ERR_DTYPE;
    if (d->dH_dtype == CCE_BF16 && d->in_dtype != CCE_BF16) return CCE_ERR_DTYPE;
    if (d->algo != CCE_ALGO_AUTO && d->algo != CCE_ALGO_GATHER && d->algo != CCE_ALGO_TILE) return CCE_ERR_UNSUPPORTED;
    if (d->algo == CCE_ALGO_TILE && !tile_eligible(d)) return CCE_ERR_UNSUPPORTED;
    if (!(d->filter_eps >= 0.f)) return CCE_ERR_SHAPE;  // negative or NaN
    if (d->filter_eps > 0.f && !(d->neg_mode == CCE_NEG_FULL && use_tile(d))) return CCE_ERR_UNSUPPORTED;
    return CCE_OK;
}

cce_status check_common(const cce_desc *d, const void *H, const void *E, const int32_t *tgt, const int32_t *neg,
                        void *workspace, size_t workspace_bytes)
{
    const cce_status st = check_desc(d);
    if (st != CCE_OK) return st;
    if (!H || !E || !tgt) return CCE_ERR_NULL;
    if (d->neg_mode != CCE_NEG_FULL && d->K > 0 && !neg) return CCE_ERR_NULL;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 15u) || workspace_bytes < cce_neg_workspace_bytes(d))
        return CCE_ERR_WORKSPACE;
    return CCE_OK;
}

Params make_params(const cce_desc *d, const void *H, const void *E, const int32_t *tgt, const int32_t *neg,
                   const uint8_t *mask, void *workspace)
{
    Params p{};
    p.H = H;
    p.E = E;
    p.tgt = tgt;
    p.neg = neg;
    p.mask = mask;
    p.status = static_cast<int32_t *>(workspace);
    p.N = d->N;
    p.V = d->V;
    p.d = d->d;
    p.K = (d->neg_mode == CCE_NEG_FULL) ? 0 : d->K;
    p.neg_mode = d->neg_mode;
    p.collide = d->mask_target_collisions ? 1 : 0;
    p.validate = d->validate_indices ? 1 : 0;
    p.dH_bf16 = (d->dH_dtype == CCE_BF16) ? 1 : 0;
    return p;
}

// Workspace of the per-position mode: the correct-item coefficients and the inverted index of the negatives, which is
// built and used up in slices of the item-id range: 12 bytes per pair of ONE slice (at most max(2^22, N K / 8) pairs),
// one word per item, one per position, and the (bucket, block) counts of the first sort level (32 MiB at most).
struct PpLayout {
    size_t coef, cursor, block_sums, pairs, tmp, part_hist, hot_list, plan, U, total;
};
PpLayout make_pp_layout(const cce_desc *d)
{
    PpLayout L{};
    const size_t n_pairs = (size_t)invert_index_pairs(d->N, d->K);
    const bool part = invert_partitioned(d->V);
    const size_t n_buckets = part ? (size_t)invert_buckets(d->V) : 0;
    const size_t n_hist = part ? n_buckets * (size_t)invert_part_blocks(d->N, d->K) + 1 : 0;
    const size_t scan_n = part ? n_hist : (size_t)d->V;
    size_t off = kHeaderBytes;
    L.coef = off;        off += align256((size_t)d->N * 4);
    L.cursor = off;      off += align256((size_t)d->V * 4);
    L.block_sums = off;  off += align256(invert_scan_blocks((int64_t)scan_n) * 4);
    L.pairs = off;       off += align256(n_pairs * 4);
    L.tmp = off;         off += part ? align256(n_pairs * 8) : 0;
    L.part_hist = off;   off += align256(n_hist * 4);
    L.hot_list = off;    off += align256(invert_hot_capacity(d->N, d->K) * 16);
    L.plan = off;        off += align256((2 * n_buckets + (size_t)invert_plan_words()) * 4);
    L.U = off;           off += d->fuse_dH ? align256((size_t)d->N * (size_t)d->d * 4) : 0;  // fused forward pass
    L.total = off;
    return L;
}
bool use_inverted(const cce_desc *d)
{
    // The index holds 32-bit offsets: larger problems keep the atomic row adds of the row-gather pass, and so do
    // catalogues beyond the sliced build (more than 2048 * 2048 items) whose pairs do not fit one slice.
    if (d->neg_mode != CCE_NEG_PER_POSITION || d->K <= 0 || d->N * (int64_t)d->K >= 0x7fffffffLL) return false;
    return invert_partitioned(d->V) || invert_slices(d->N, d->K) == 1;
}

// The forward call of the row-gather family forms the hidden-state gradient as well (fuse_dH): every mode but
// per-position negatives too many for the inverted index (their backward pass gathers the rows anyway, for dE).
bool fused_gather(const cce_desc *d)
{
    return d->fuse_dH != 0 && !use_tile(d) && (d->neg_mode != CCE_NEG_PER_POSITION || use_inverted(d));
}
// ... and what it keeps in the workspace where there is no inverted index: p+ - 1 per position and the rows U.
struct PlainLayout {
    size_t coef, U, total;
};
PlainLayout make_plain_layout(const cce_desc *d)
{
    PlainLayout L{};
    size_t off = kHeaderBytes;
    L.coef = off;  off += align256((size_t)d->N * 4);
    L.U = off;     off += align256((size_t)d->N * (size_t)d->d * 4);
    L.total = off;
    return L;
}
void set_fused_gather(const cce_desc *d, void *workspace, Params &p)
{
    char *ws = static_cast<char *>(workspace);
    if (use_inverted(d)) {
        const PpLayout L = make_pp_layout(d);
        p.coef = reinterpret_cast<float *>(ws + L.coef);
        p.U = reinterpret_cast<float *>(ws + L.U);
    } else {
        const PlainLayout L = make_plain_layout(d);
        p.coef = reinterpret_cast<float *>(ws + L.coef);
        p.U = reinterpret_cast<float *>(ws + L.U);
    }
}

TileArgs make_tile_args(const cce_desc *d, const Layout &L, const void *H, const void *E, const int32_t *tgt,
                        const int32_t *neg, const uint8_t *mask, void *workspace)
{
    char *ws = static_cast<char *>(workspace);
    int32_t *header = static_cast<int32_t *>(workspace);
    const bool compact = (mask != nullptr) || d->validate_indices;
    const bool shared = (d->neg_mode == CCE_NEG_SHARED);
    TileArgs a{};
    a.H = static_cast<const uint16_t *>(H);
    a.E = static_cast<const uint16_t *>(E);
    a.tgt = tgt;
    a.neg = shared ? neg : nullptr;
    a.idx = compact ? reinterpret_cast<const int32_t *>(ws + L.idx) : nullptr;
    a.n_valid_ptr = compact ? header + kHdrNValid : nullptr;
    a.cnt = (shared && d->mask_target_collisions) ? reinterpret_cast<const int32_t *>(ws + L.cnt) : nullptr;
    a.coef = reinterpret_cast<float *>(ws + L.coef);
    a.de_const = reinterpret_cast<uint32_t *>(ws + L.de_const);
    a.part_m = reinterpret_cast<float *>(ws + L.part_m);
    a.part_s = reinterpret_cast<float *>(ws + L.part_s);
    a.part_dH = reinterpret_cast<float *>(ws + L.part_dH);
    a.U = fused_dH(d) ? reinterpret_cast<float *>(ws + L.U) : nullptr;
    a.N = d->N;
    a.V = d->V;
    a.n_cols = shared ? d->K : d->V;
    a.d = d->d;
    a.splits = L.splits_x;
    a.pos_weight_mode = shared ? 0 : 2;
    a.dH_bf16 = (d->dH_dtype == CCE_BF16) ? 1 : 0;
    a.validate = d->validate_indices ? 1 : 0;
    return a;
}

PrepArgs make_prep_args(const cce_desc *d, const Layout &L, const int32_t *tgt, const int32_t *neg,
                        const uint8_t *mask, void *workspace)
{
    char *ws = static_cast<char *>(workspace);
    const bool compact = (mask != nullptr) || d->validate_indices;
    const bool shared = (d->neg_mode == CCE_NEG_SHARED);
    PrepArgs p{};
    p.tgt = tgt;
    p.neg = shared ? neg : nullptr;
    p.mask = mask;
    p.header = static_cast<int32_t *>(workspace);
    p.idx = compact ? reinterpret_cast<int32_t *>(ws + L.idx) : nullptr;
    p.cnt = (shared && d->mask_target_collisions) ? reinterpret_cast<int32_t *>(ws + L.cnt) : nullptr;
    p.N = d->N;
    p.V = d->V;
    p.d = d->d;
    p.K = shared ? d->K : 0;
    p.validate = d->validate_indices ? 1 : 0;
    p.dH_bf16 = (d->dH_dtype == CCE_BF16) ? 1 : 0;
    return p;
}

// What a forward call alone touches of the workspace: everything in front of the partial dH rows on the matrix-core
// path, the header otherwise (the inverted index and the coefficients of the per-position layout are the backward
// call's).
size_t forward_scratch_bytes(const cce_desc *d)
{
    return use_tile(d) ? make_layout(d).part_dH : kHeaderBytes;
}

// Shared mode: the sampled calls write their K ids behind everything else in the workspace.
size_t shared_ids_offset(const cce_desc *d)
{
    if (use_tile(d)) return make_layout(d).total;
    if (use_inverted(d)) return make_pp_layout(d).total;
    return fused_gather(d) ? make_plain_layout(d).total : kHeaderBytes;
}

cce_status check_sampler(const cce_desc *d, const cce_sampler *s)
{
    const cce_status st = check_desc(d);
    if (st != CCE_OK) return st;
    if (!s) return CCE_ERR_NULL;
    if (d->neg_mode == CCE_NEG_FULL) return CCE_ERR_UNSUPPORTED;
    if (s->kind != CCE_SAMPLER_UNIFORM && s->kind != CCE_SAMPLER_ALIAS) return CCE_ERR_SHAPE;
    if (s->kind == CCE_SAMPLER_ALIAS && (!s->alias_thresh || !s->alias_id)) return CCE_ERR_NULL;
    return CCE_OK;
}

Sampler make_sampler(const cce_desc *d, const cce_sampler *s)
{
    Sampler r{};
    r.kind = (uint32_t)s->kind;
    r.k0 = (uint32_t)(s->seed & 0xffffffffu);
    r.k1 = (uint32_t)(s->seed >> 32);
    r.stream = s->stream;
    r.V = (uint32_t)d->V;
    r.thresh = s->alias_thresh;
    r.alias = s->alias_id;
    return r;
}

}  // namespace

// ---- profiling records
namespace {
struct ProfRecord {
    int family;
    hipEvent_t start, stop;
};
bool g_prof_enabled = false;
std::vector<ProfRecord> g_prof_records;
std::vector<hipEvent_t> g_prof_pool;
const char *const kProfNames[PROF_FAMILIES] = {"gather_fwd", "gather_bwd", "prep",  "tile_fwd", "fwd_merge",  "tile_dh",
                                               "dh_merge",   "tile_de",    "index", "item_de",  "pos_scatter", "bwd_pre", "tile_bwd",
                                               "tile_fdh",   "fdh_merge",  "dh_scale"};
hipEvent_t prof_event()
{
    if (!g_prof_pool.empty()) {
        hipEvent_t e = g_prof_pool.back();
        g_prof_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
}  // namespace

ProfScope::ProfScope(int family, hipStream_t s) : slot(-1), stream(s)
{
    if (!g_prof_enabled) return;
    ProfRecord r{family, prof_event(), prof_event()};
    if (!r.start || !r.stop) return;
    (void)hipEventRecord(r.start, stream);
    g_prof_records.push_back(r);
    slot = (int)g_prof_records.size() - 1;
}
ProfScope::~ProfScope()
{
    if (slot >= 0) (void)hipEventRecord(g_prof_records[slot].stop, stream);
}

hipError_t launch_fill_zero(int32_t *dst, size_t words, hipStream_t stream)
{
    if (words == 0) return hipSuccess;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, stream, dst, words);
    return hipGetLastError();
}

}  // namespace cce

extern "C" {

size_t cce_neg_workspace_bytes(const cce_desc *desc)
{
    if (cce::check_desc(desc) != CCE_OK) return 0;
    return cce::shared_ids_offset(desc) + (desc->neg_mode == CCE_NEG_SHARED ? cce::align256((size_t)desc->K * 4) : 0);
}

cce_status cce_neg_workspace_init(void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!workspace) return CCE_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(workspace) & 15u) || workspace_bytes < cce::kHeaderBytes) return CCE_ERR_WORKSPACE;
    const hipError_t e = cce::launch_fill_zero(static_cast<int32_t *>(workspace), cce::kHeaderBytes / 4,
                                               static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? CCE_OK : CCE_ERR_HIP;
}

}  // extern "C"

// ---- scratch of the entry point that takes no workspace: one array per GPU, held until the process ends
namespace cce {
namespace {
constexpr size_t kStaticScratchBytes = size_t(32) << 20;
}
}  // namespace cce
// In host code this name only stands for the symbol; its device address comes from hipGetSymbolAddress (below).
static __device__ __align__(256) unsigned char scratch[cce::kStaticScratchBytes];

namespace cce {
namespace {

// Device address of `scratch` on the current device, looked up once per device (every GPU holds its own copy of the
// array at its own address) and kept.  Not an allocation: the array is part of the library's code object.
cce_status static_scratch(void **out)
{
    static std::mutex lock;
    static void *ptr[kMaxScratchDevices];  // nullptr = not looked up yet
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxScratchDevices) return CCE_ERR_HIP;
    std::lock_guard<std::mutex> hold(lock);
    if (!ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return CCE_ERR_HIP;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return CCE_OK;
}

// Shared mode of the sampled calls: draw the K ids into the workspace and hand them on as a stored list.
// Per-position mode: the kernels draw; `neg` stays NULL.
cce_status stage_sampler(const cce_desc *desc, const cce_sampler *sampler, void *workspace, hipStream_t stream,
                         const int32_t *&neg, Sampler &smp, bool ids_still_there = false)
{
    smp = Sampler{};
    neg = nullptr;
    if (desc->K == 0) return CCE_OK;
    const Sampler s = make_sampler(desc, sampler);
    if (desc->neg_mode == CCE_NEG_SHARED) {
        int32_t *ids = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + shared_ids_offset(desc));
        if (!ids_still_there && launch_sample(s, 1, desc->K, ids, stream) != hipSuccess) return CCE_ERR_HIP;
        neg = ids;
    } else {
        smp = s;
    }
    return CCE_OK;
}

cce_status forward_impl(const cce_desc *desc, const Sampler &smp, const void *H, const void *E, const int32_t *tgt,
                        const int32_t *neg, const uint8_t *mask, float *loss, float *lse, void *workspace,
                        hipStream_t stream)
{
    if (cce::use_tile(desc)) {
        const cce::Layout L = cce::make_layout(desc);
        cce::PrepArgs pa = cce::make_prep_args(desc, L, tgt, neg, mask, workspace);
        pa.loss = loss;
        pa.lse = lse;
        if (pa.idx || pa.cnt) {
            if (cce::launch_prep(pa, stream) != hipSuccess) return CCE_ERR_HIP;
        }
        cce::TileArgs a = cce::make_tile_args(desc, L, H, E, tgt, neg, mask, workspace);
        a.loss = loss;
        a.lse = lse;
        if (cce::fused_dH(desc)) {  // lse and the hidden-state gradient short of grad_loss in one pass (splits as the dH pass)
            a.splits = L.splits_x;
            return cce::launch_tile(cce::TILE_PASS_FDH, a, stream) == hipSuccess ? CCE_OK : CCE_ERR_HIP;
        }
        a.splits = L.splits_fwd;
        return cce::launch_tile(cce::TILE_PASS_FWD, a, stream) == hipSuccess ? CCE_OK : CCE_ERR_HIP;
    }
    cce::Params p = cce::make_params(desc, H, E, tgt, neg, mask, workspace);
    p.loss = loss;
    p.lse = lse;
    p.smp = smp;
    if (cce::fused_gather(desc)) cce::set_fused_gather(desc, workspace, p);  // the kernel that also files U and p+ - 1
    const hipError_t e = cce::launch_gather(false, desc->in_dtype == CCE_BF16, p, stream);
    return e == hipSuccess ? CCE_OK : CCE_ERR_HIP;
}

cce_status backward_impl(const cce_desc *desc, const Sampler &smp, const void *H, const void *E, const int32_t *tgt,
                         const int32_t *neg, const uint8_t *mask, const float *lse, const float *grad_loss, void *dH,
                         float *dE, void *workspace, hipStream_t stream)
{
    if (cce::use_tile(desc)) {
        const cce::Layout L = cce::make_layout(desc);
        cce::PrepArgs pa = cce::make_prep_args(desc, L, tgt, neg, mask, workspace);
        // The compaction and the collision counts depend on tgt, neg and mask only: a caller that vouches for the
        // workspace still holding what the forward call left there spares their recomputation.
        if ((pa.idx || pa.cnt) && !desc->reuse_forward_prep) {
            if (cce::launch_prep(pa, stream) != hipSuccess) return CCE_ERR_HIP;
        }
        cce::TileArgs a = cce::make_tile_args(desc, L, H, E, tgt, neg, mask, workspace);
        a.pos_mask = mask;  // the dH launch zeroes the rows of padded positions itself
        a.lse_in = lse;
        a.g = grad_loss;
        a.dH = dH;
        a.dE = dE;
        a.write_consts = 1;
        a.filter_log2 = desc->filter_eps > 0.f ? log2f(desc->filter_eps) : -INFINITY;
        // The forward call leaves the per-position constants of the backward pass that do not involve the upstream
        // gradient; a caller who vouches for the workspace spares the pass that would recompute them.
        a.g_separate = (desc->reuse_forward_prep && grad_loss && cce::tile_backward_fusable(desc->d)) ? 1 : 0;
        cce::TileArgs a_de = a;
        a_de.splits = L.splits_de;
        if (cce::fused_dH(desc) && desc->reuse_forward_prep && !(desc->filter_eps > 0.f)) {
            // The forward call left U, the correct items' coefficients and the exponent offsets of the dE pass: dH is
            // grad_loss * U, and the scores are recomputed for dE alone.  Where the dE pass streams grad_loss by row
            // number (hidden sizes up to 128, grad_loss given) the scaling rides in its launch; otherwise it goes first
            // and files grad_loss under the compacted index on the way.
            a_de.g_separate = 1;  // the scatter multiplies the forward call's coefficient by grad_loss itself
            if (cce::tile_backward_fusable(desc->d) && grad_loss) {
                a_de.scale_blocks = 1;
                return cce::launch_tile(cce::TILE_PASS_DE, a_de, stream) == hipSuccess ? CCE_OK : CCE_ERR_HIP;
            }
            a_de.g_stream_off = 1;  // the dE pass reads grad_loss where the scaling pass has filed it
            if (cce::tile_backward_fusable(desc->d)) {  // no grad_loss array to stream: scale (and file ones) first
                if (cce::launch_dh_scale(a, true, stream) != hipSuccess) return CCE_ERR_HIP;
            } else {
                a_de.scale_blocks = 1;  // hidden size 256: the scaling shares the launch of the correct-item scatter
            }
            return cce::launch_tile(cce::TILE_PASS_DE, a_de, stream) == hipSuccess ? CCE_OK : CCE_ERR_HIP;
        }
        if (cce::tile_backward_fusable(desc->d))  // both passes in one launch, behind a small per-position pass
            return cce::launch_tile_backward(a, a_de, stream) == hipSuccess ? CCE_OK : CCE_ERR_HIP;
        if (cce::launch_tile(cce::TILE_PASS_DH, a, stream) != hipSuccess) return CCE_ERR_HIP;
        return cce::launch_tile(cce::TILE_PASS_DE, a_de, stream) == hipSuccess ? CCE_OK : CCE_ERR_HIP;
    }
    cce::Params p = cce::make_params(desc, H, E, tgt, neg, mask, workspace);
    p.lse_in = lse;
    p.g = grad_loss;
    p.dH = dH;
    p.dE = dE;
    p.smp = smp;
    const bool bf16 = desc->in_dtype == CCE_BF16;
    const bool scatter = bf16 && cce::tile_supports_d(desc->d);  // the aggregated scatter of the correct items exists
    // fuse_dH: the forward call left U and p+ - 1; no candidate row is gathered for dH
    const bool fused = cce::fused_gather(desc) && desc->reuse_forward_prep;
    cce::TileArgs t{};
    if (scatter) {
        t.H = static_cast<const uint16_t *>(H);
        t.tgt = tgt;
        t.pos_mask = mask;
        t.dE = dE;
        t.N = desc->N;
        t.V = desc->V;
        t.d = desc->d;
        t.validate = desc->validate_indices ? 1 : 0;
    }
    if (fused) {
        cce::set_fused_gather(desc, workspace, p);
        if (cce::launch_gather_scale(bf16, !scatter, p, stream) != hipSuccess) return CCE_ERR_HIP;
        t.coef = p.coef;       // short of the upstream gradient:
        t.g_separate = 1;      // the scatter multiplies by grad_loss itself
        t.g = grad_loss;
    }
    if (!cce::use_inverted(desc)) {
        // Shared negatives or the full catalogue: the position-major pass yields dH and the correct items' dE rows; the
        // rows of the shared candidates, which every position updates, come from a candidate-major pass.
        const bool shared_rows = desc->neg_mode != CCE_NEG_PER_POSITION;
        if (fused) {  // (never per-position here)
            if (scatter && cce::launch_pos_scatter(t, stream) != hipSuccess) return CCE_ERR_HIP;
            return cce::launch_shared_dE(bf16, p, stream) == hipSuccess ? CCE_OK : CCE_ERR_HIP;
        }
        if (shared_rows) p.skip_neg_dE = 1;
        if (cce::launch_gather(true, desc->in_dtype == CCE_BF16, p, stream) != hipSuccess) return CCE_ERR_HIP;
        if (shared_rows && cce::launch_shared_dE(desc->in_dtype == CCE_BF16, p, stream) != hipSuccess) return CCE_ERR_HIP;
        return CCE_OK;
    }
    // Per-position negatives: the row-gather pass yields dH and the correct-item coefficients; dE of the negatives
    // comes from the inverted-index pass, dE of the correct items from the aggregated scatter where it exists.
    const cce::PpLayout L = cce::make_pp_layout(desc);
    char *ws = static_cast<char *>(workspace);
    if (!fused) {
        p.skip_neg_dE = 1;
        p.skip_pos_dE = scatter ? 1 : 0;
        p.coef = reinterpret_cast<float *>(ws + L.coef);
        if (cce::launch_gather(true, bf16, p, stream) != hipSuccess) return CCE_ERR_HIP;
        t.coef = p.coef;
    }
    cce::InvertArgs ia{};
    ia.H = H;
    ia.E = E;
    ia.tgt = tgt;
    ia.neg = neg;
    ia.mask = mask;
    ia.lse_in = lse;
    ia.g = grad_loss;
    ia.dE = dE;
    ia.cursor = reinterpret_cast<int32_t *>(ws + L.cursor);
    ia.block_sums = reinterpret_cast<int32_t *>(ws + L.block_sums);
    ia.pairs = reinterpret_cast<int32_t *>(ws + L.pairs);
    ia.tmp = reinterpret_cast<int2 *>(ws + L.tmp);
    ia.part_hist = reinterpret_cast<int32_t *>(ws + L.part_hist);
    ia.hot_list = reinterpret_cast<int4 *>(ws + L.hot_list);
    ia.bucket_start = reinterpret_cast<int32_t *>(ws + L.plan);
    const int64_t n_buckets = cce::invert_partitioned(desc->V) ? cce::invert_buckets(desc->V) : 0;
    ia.slice_of = ia.bucket_start + n_buckets;
    ia.slice_hot = ia.slice_of + n_buckets;
    ia.hot_count = static_cast<int32_t *>(workspace) + cce::kHdrHot;
    ia.hot_capacity = (int32_t)cce::invert_hot_capacity(desc->N, desc->K);
    ia.N = desc->N;
    ia.V = desc->V;
    ia.d = desc->d;
    ia.K = desc->K;
    ia.collide = desc->mask_target_collisions ? 1 : 0;
    ia.validate = desc->validate_indices ? 1 : 0;
    ia.smp = smp;
    return cce::launch_inverted_dE(bf16, ia, scatter ? &t : nullptr, stream) == hipSuccess ? CCE_OK : CCE_ERR_HIP;
}

}  // namespace
}  // namespace cce

extern "C" {

cce_status cce_neg_forward(const cce_desc *desc, const void *H, const void *E, const int32_t *tgt, const int32_t *neg,
                           const uint8_t *mask, float *loss, float *lse, void *workspace, size_t workspace_bytes,
                           void *hip_stream)
{
    const cce_status st = cce::check_common(desc, H, E, tgt, neg, workspace, workspace_bytes);
    if (st != CCE_OK) return st;
    if (!loss || !lse) return CCE_ERR_NULL;
    return cce::forward_impl(desc, cce::Sampler{}, H, E, tgt, neg, mask, loss, lse, workspace,
                             static_cast<hipStream_t>(hip_stream));
}

cce_status cce_neg_backward(const cce_desc *desc, const void *H, const void *E, const int32_t *tgt, const int32_t *neg,
                            const uint8_t *mask, const float *lse, const float *grad_loss, void *dH, float *dE,
                            void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const cce_status st = cce::check_common(desc, H, E, tgt, neg, workspace, workspace_bytes);
    if (st != CCE_OK) return st;
    if (!lse || !dH || !dE) return CCE_ERR_NULL;
    return cce::backward_impl(desc, cce::Sampler{}, H, E, tgt, neg, mask, lse, grad_loss, dH, dE, workspace,
                              static_cast<hipStream_t>(hip_stream));
}

cce_status cce_neg_forward_noalloc(const cce_desc *desc, const void *H, const void *E, const int32_t *tgt,
                                   const int32_t *neg, const uint8_t *mask, float *loss, float *lse, void *hip_stream)
{
    cce_status st = cce::check_desc(desc);
    if (st != CCE_OK) return st;
    if (!H || !E || !tgt || !loss || !lse) return CCE_ERR_NULL;
    if (desc->neg_mode != CCE_NEG_FULL && desc->K > 0 && !neg) return CCE_ERR_NULL;
    if (desc->validate_indices) return CCE_ERR_UNSUPPORTED;  // no status word the caller could read afterwards
    if (desc->fuse_dH) return CCE_ERR_UNSUPPORTED;           // the rows it would keep belong in a caller-owned workspace
    if (cce::forward_scratch_bytes(desc) > cce::kStaticScratchBytes) return CCE_ERR_WORKSPACE;
    void *ws = nullptr;
    st = cce::static_scratch(&ws);
    if (st != CCE_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // the array keeps what the last call left: the header (status word, counters) starts from zero every time
    if (cce::launch_fill_zero(static_cast<int32_t *>(ws), cce::kHeaderBytes / 4, stream) != hipSuccess) return CCE_ERR_HIP;
    return cce::forward_impl(desc, cce::Sampler{}, H, E, tgt, neg, mask, loss, lse, ws, stream);
}

cce_status cce_neg_sample(const cce_desc *desc, const cce_sampler *sampler, int32_t *neg_out, void *hip_stream)
{
    const cce_status st = cce::check_sampler(desc, sampler);
    if (st != CCE_OK) return st;
    if (desc->K > 0 && !neg_out) return CCE_ERR_NULL;
    const int64_t n_pos = (desc->neg_mode == CCE_NEG_SHARED) ? 1 : desc->N;
    const hipError_t e = cce::launch_sample(cce::make_sampler(desc, sampler), n_pos, desc->K, neg_out,
                                            static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? CCE_OK : CCE_ERR_HIP;
}

cce_status cce_neg_forward_sampled(const cce_desc *desc, const cce_sampler *sampler, const void *H, const void *E,
                                   const int32_t *tgt, const uint8_t *mask, float *loss, float *lse, void *workspace,
                                   size_t workspace_bytes, void *hip_stream)
{
    cce_status st = cce::check_sampler(desc, sampler);
    if (st != CCE_OK) return st;
    int32_t stand_in = 0;  // the common checks only ask that a list exists when K > 0
    st = cce::check_common(desc, H, E, tgt, &stand_in, workspace, workspace_bytes);
    if (st != CCE_OK) return st;
    if (!loss || !lse) return CCE_ERR_NULL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int32_t *neg;
    cce::Sampler smp;
    st = cce::stage_sampler(desc, sampler, workspace, stream, neg, smp);
    if (st != CCE_OK) return st;
    return cce::forward_impl(desc, smp, H, E, tgt, neg, mask, loss, lse, workspace, stream);
}

cce_status cce_neg_backward_sampled(const cce_desc *desc, const cce_sampler *sampler, const void *H, const void *E,
                                    const int32_t *tgt, const uint8_t *mask, const float *lse, const float *grad_loss,
                                    void *dH, float *dE, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    cce_status st = cce::check_sampler(desc, sampler);
    if (st != CCE_OK) return st;
    int32_t stand_in = 0;
    st = cce::check_common(desc, H, E, tgt, &stand_in, workspace, workspace_bytes);
    if (st != CCE_OK) return st;
    if (!lse || !dH || !dE) return CCE_ERR_NULL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int32_t *neg;
    cce::Sampler smp;
    // reuse_forward_prep: the list the forward call drew is still in the workspace
    st = cce::stage_sampler(desc, sampler, workspace, stream, neg, smp, desc->reuse_forward_prep != 0);
    if (st != CCE_OK) return st;
    return cce::backward_impl(desc, smp, H, E, tgt, neg, mask, lse, grad_loss, dH, dE, workspace, stream);
}

cce_status cce_neg_index_status(void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!workspace) return CCE_ERR_NULL;
    if (workspace_bytes < cce::kHeaderBytes) return CCE_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int32_t word = 0;
    if (hipMemcpyAsync(&word, workspace, sizeof word, hipMemcpyDeviceToHost, s) != hipSuccess) return CCE_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return CCE_ERR_HIP;
    if (word != 0) {
        if (cce::launch_fill_zero(static_cast<int32_t *>(workspace), 1, s) != hipSuccess) return CCE_ERR_HIP;
        if (hipStreamSynchronize(s) != hipSuccess) return CCE_ERR_HIP;
        return CCE_ERR_INDEX;
    }
    return CCE_OK;
}

cce_status cce_neg_profile_enable(int32_t enable)
{
    cce::g_prof_enabled = enable != 0;
    return CCE_OK;
}

int32_t cce_neg_profile_read(int32_t max, char *names, float *total_ms, int32_t *launches)
{
    float sum[cce::PROF_FAMILIES] = {};
    int32_t cnt[cce::PROF_FAMILIES] = {};
    for (const cce::ProfRecord &r : cce::g_prof_records) {
        float ms = 0.f;
        if (hipEventSynchronize(r.stop) == hipSuccess && hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
            sum[r.family] += ms;
            cnt[r.family] += 1;
        }
        cce::g_prof_pool.push_back(r.start);
        cce::g_prof_pool.push_back(r.stop);
    }
    cce::g_prof_records.clear();
    int32_t n = 0;
    for (int f = 0; f < cce::PROF_FAMILIES && n < max; ++f) {
        if (cnt[f] == 0) continue;
        if (names) {
            strncpy(names + (size_t)n * 32, cce::kProfNames[f], 31);
            names[(size_t)n * 32 + 31] = 0;
        }
        if (total_ms) total_ms[n] = sum[f];
        if (launches) launches[n] = cnt[f];
        ++n;
    }
    return n;
}

const char *cce_status_string(cce_status status)
{
    switch (status) {
    case CCE_OK: return "ok";
    case CCE_ERR_NULL: return "a required pointer is NULL";
    case CCE_ERR_SHAPE: return "invalid shape (N, V, K, d or neg_mode)";
    case CCE_ERR_DTYPE: return "invalid dtype combination";
    case CCE_ERR_INDEX: return "an id of a valid position is outside [0, V)";
    case CCE_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case CCE_ERR_UNSUPPORTED: return "requested algorithm cannot run this descriptor";
    case CCE_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

}  // extern "C"
