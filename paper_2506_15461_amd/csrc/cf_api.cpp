// Host side of the C ABI declared in include/checkfree.h: handles, validation,
// chunk planning, launch-shape selection.  No arithmetic of the method lives
// here; every step of the path runs in the kernels of cf_kernels.hip.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "checkfree.h"
#include "cf_kernels.h"

namespace {

constexpr uint32_t kDefaultChunkBytes = 128u << 10;   // 128 tiles of 1 KiB
constexpr uint32_t kMinChunkBytes = 4096;
constexpr uint32_t kMaxChunkBytes = 4u << 20;
constexpr uint32_t kDefaultSqnormBlocksPerCu = 0;     // 0: the measured best (kCappedGridPerCu)
constexpr uint32_t kOnePerChunk = 65;                 // tuning value that forces one workgroup per chunk
constexpr uint32_t kCappedGridPerCu = 2;
constexpr uint64_t kMaxChunksPerStage = 1ull << 31;
constexpr uint64_t kMaxGrid = (1ull << 31) - 1;
constexpr size_t kCtxWordBytes = CF_CTX_WORDS * sizeof(uint32_t);
constexpr uint64_t kTableAlign = 256;   // sections of a stage's device tables start on multiples of this

std::atomic<uint64_t> g_next_stage_id{1};

uint32_t elem_size(int32_t dtype) { return dtype == CF_F32 ? 4u : 2u; }

struct HostTensor {
    uint64_t addr;
    uint64_t numel;
    int32_t dtype;
};

}  // namespace

struct cf_ctx {
    int device = 0;
    int num_cu = 0;
    cf_tuning tuning{};
    uint32_t tile_shift = 0;   // log2(chunk_bytes / CF_TILE_BYTES)
    uint32_t *d_words = nullptr;
    bool owns_words = false;   // d_words came from hipMalloc here (else it is the caller's workspace)
    void *d_static = nullptr;  // this device's copy of the library's static scratch array
    std::atomic<uint32_t> live_stages{0};
    // Pairs (input stage id, output stage id) whose congruence and aliasing have been checked.
    std::mutex checked_mutex;
    std::vector<std::pair<uint64_t, uint64_t>> checked;
};

struct cf_stage {
    cf_ctx *ctx = nullptr;
    uint64_t id = 0;
    std::vector<HostTensor> tensors;
    uint64_t numel = 0;
    uint64_t nbytes = 0;
    uint32_t n_chunks = 0;
    void *d_table = nullptr;       // the device block the three tables below live in
    bool owns_table = false;       // d_table came from hipMalloc here (else it is the caller's)
    CfChunk *d_chunks = nullptr;   // n_chunks entries
    double *d_partials = nullptr;  // n_chunks doubles (sqnorm scratch)
    uint32_t *d_tensor_first = nullptr;   // tensors + 1 entries: first chunk of each tensor
};

namespace {

class DeviceGuard {
public:
    explicit DeviceGuard(int device) : ok_(false), prev_(0)
    {
        if (hipGetDevice(&prev_) != hipSuccess) return;
        if (prev_ != device && hipSetDevice(device) != hipSuccess) return;
        ok_ = true;
        changed_ = prev_ != device;
    }
    ~DeviceGuard()
    {
        if (ok_ && changed_) (void)hipSetDevice(prev_);
    }
    bool ok() const { return ok_; }

private:
    bool ok_;
    bool changed_ = false;
    int prev_;
};

cf_status check_tensor(const cf_tensor &t)
{
    if (t.dtype != CF_F32 && t.dtype != CF_BF16) return CF_ERR_DTYPE;
    if (t.numel != 0 && t.data == nullptr) return CF_ERR_NULL;
    if (t.numel != 0 && (reinterpret_cast<uint64_t>(t.data) % elem_size(t.dtype)) != 0) return CF_ERR_ALIGN;
    if (t.numel > (1ull << 40)) return CF_ERR_LIMIT;
    return CF_OK;
}

uint64_t chunks_of(uint64_t numel, uint64_t chunk_elems) { return (numel + chunk_elems - 1) / chunk_elems; }

uint64_t align_up(uint64_t v) { return (v + kTableAlign - 1) / kTableAlign * kTableAlign; }

// Where a stage's three tables sit inside its device block.
struct TableLayout {
    uint64_t chunks_off, first_off, partials_off, total;
};

TableLayout table_layout(uint64_t n_chunks, uint32_t num_tensors)
{
    TableLayout l;
    l.chunks_off = 0;
    l.first_off = align_up(n_chunks * sizeof(CfChunk));
    l.partials_off = l.first_off + (num_tensors ? align_up(((uint64_t)num_tensors + 1) * sizeof(uint32_t)) : 0);
    l.total = l.partials_off + align_up(n_chunks * sizeof(double));
    return l;
}

// Validates a tensor list and counts its chunks.
cf_status plan_stage(const cf_ctx *ctx, const cf_tensor *tensors, uint32_t num_tensors, uint64_t *n_chunks_out)
{
    const uint32_t chunk_bytes = ctx->tuning.chunk_bytes;
    uint64_t n_chunks = 0;
    for (uint32_t t = 0; t < num_tensors; ++t) {
        cf_status st = check_tensor(tensors[t]);
        if (st != CF_OK) return st;
        n_chunks += chunks_of(tensors[t].numel, chunk_bytes / elem_size(tensors[t].dtype));
    }
    if (n_chunks >= kMaxChunksPerStage || (n_chunks << ctx->tile_shift) > kMaxGrid) return CF_ERR_LIMIT;
    *n_chunks_out = n_chunks;
    return CF_OK;
}

bool valid_chunk_bytes(uint32_t b)
{
    return b >= kMinChunkBytes && b <= kMaxChunkBytes && (b & (b - 1)) == 0;
}

struct Range {
    uint64_t lo, hi;
    uint32_t index;
};

// `out` may coincide with `in` tensor for tensor; any other shared byte is an error.
cf_status check_pair(const std::vector<HostTensor> &in, const std::vector<HostTensor> &out)
{
    if (in.size() != out.size()) return CF_ERR_SHAPE_MISMATCH;
    const size_t n = in.size();
    for (size_t t = 0; t < n; ++t) {
        if (in[t].numel != out[t].numel || in[t].dtype != out[t].dtype) return CF_ERR_SHAPE_MISMATCH;
    }
    // Sweep over the input ranges sorted by address; for each output range look at its neighbours.
    std::vector<Range> rin;
    rin.reserve(n);
    for (size_t t = 0; t < n; ++t) {
        const HostTensor &h = in[t];
        if (h.numel) rin.push_back({h.addr, h.addr + h.numel * elem_size(h.dtype), (uint32_t)t});
    }
    std::sort(rin.begin(), rin.end(), [](const Range &x, const Range &y) { return x.lo < y.lo; });
    // Input ranges may themselves overlap (a tensor listed twice); keep a running maximum of `hi`.
    std::vector<uint64_t> max_hi(rin.size());
    uint64_t m = 0;
    for (size_t i = 0; i < rin.size(); ++i) {
        m = std::max(m, rin[i].hi);
        max_hi[i] = m;
    }
    for (size_t t = 0; t < n; ++t) {
        const HostTensor &o = out[t];
        if (!o.numel) continue;
        const uint64_t lo = o.addr, hi = o.addr + o.numel * elem_size(o.dtype);
        // first input range with lo >= hi of the output: everything from there on is clear
        size_t end = std::lower_bound(rin.begin(), rin.end(), hi,
                                      [](const Range &r, uint64_t v) { return r.lo < v; }) - rin.begin();
        for (size_t i = end; i-- > 0;) {
            if (max_hi[i] <= lo) break;   // nothing at or before i reaches the output range
            if (rin[i].hi > lo) {
                const bool same = rin[i].index == t && rin[i].lo == lo && rin[i].hi == hi;
                if (!same) return CF_ERR_ALIAS;
            }
        }
    }
    return CF_OK;
}

// Output tensors must not overlap one another either (two writers of one byte).
cf_status check_self(const std::vector<HostTensor> &out)
{
    std::vector<Range> r;
    for (size_t t = 0; t < out.size(); ++t) {
        const HostTensor &h = out[t];
        if (h.numel) r.push_back({h.addr, h.addr + h.numel * elem_size(h.dtype), (uint32_t)t});
    }
    std::sort(r.begin(), r.end(), [](const Range &x, const Range &y) { return x.lo < y.lo; });
    for (size_t i = 1; i < r.size(); ++i)
        if (r[i].lo < r[i - 1].hi) return CF_ERR_ALIAS;
    return CF_OK;
}

cf_status checked_pair(cf_ctx *ctx, const cf_stage *in, const cf_stage *out)
{
    const std::pair<uint64_t, uint64_t> key(in->id, out->id);
    std::lock_guard<std::mutex> lock(ctx->checked_mutex);
    if (std::find(ctx->checked.begin(), ctx->checked.end(), key) != ctx->checked.end()) return CF_OK;
    try {
        cf_status st = check_pair(in->tensors, out->tensors);
        if (st != CF_OK) return st;
        st = check_self(out->tensors);
        if (st != CF_OK) return st;
        if (ctx->checked.size() >= 256) ctx->checked.erase(ctx->checked.begin());
        ctx->checked.push_back(key);
    } catch (...) {
        return CF_ERR_LIMIT;   // host memory exhausted
    }
    return CF_OK;
}

void forget_stage(cf_ctx *ctx, uint64_t id)
{
    std::lock_guard<std::mutex> lock(ctx->checked_mutex);
    auto &v = ctx->checked;
    v.erase(std::remove_if(v.begin(), v.end(),
                           [id](const std::pair<uint64_t, uint64_t> &p) { return p.first == id || p.second == id; }),
            v.end());
}

// Enqueues the kernels that write a stage's chunk table and first-chunk indices.  The tensor
// list travels to the device in kernel argument blocks, CF_TABLE_BATCH tensors at a time: nothing
// is copied and nothing is waited for.
hipError_t enqueue_table(const cf_ctx *ctx, const cf_tensor *tensors, uint32_t num_tensors, CfChunk *d_chunks,
                         uint32_t *d_tensor_first, uint64_t n_chunks, hipStream_t stream)
{
    const uint32_t chunk_bytes = ctx->tuning.chunk_bytes;
    CfTableArgs args;
    std::memset(&args, 0, sizeof args);
    args.chunks = d_chunks;
    args.tensor_first = d_tensor_first;
    args.chunk_bytes = chunk_bytes;
    args.end_chunk = (uint32_t)n_chunks;
    uint64_t first_chunk = 0;
    for (uint32_t t = 0; t < num_tensors; ++t) {
        const cf_tensor &d = tensors[t];
        CfTableTensor &slot = args.tensor[args.n++];
        slot.addr = reinterpret_cast<uint64_t>(d.data);
        slot.numel = d.numel;
        slot.dtype = (uint32_t)d.dtype;
        slot.first_chunk = (uint32_t)first_chunk;
        first_chunk += chunks_of(d.numel, chunk_bytes / elem_size(d.dtype));
        if (args.n == CF_TABLE_BATCH || t + 1 == num_tensors) {
            args.last = (t + 1 == num_tensors);
            hipError_t e = cf_launch_build_table(args, stream);
            if (e != hipSuccess) return e;
            args.tensor_base += args.n;
            args.n = 0;
        }
    }
    return hipSuccess;
}

// Grid of the norm's first pass.  The partials are per chunk, so the result does not depend on this
// choice; only the speed does.  Measured on this chip (cold gradients of 113 MB, 411 MB, 822 MB and
// 1.6 GB): two resident workgroups per compute unit walking the chunk list, every workgroup with the
// same number of chunks, are 1.5-3.5 % faster than one short-lived workgroup per chunk at every size;
// three or four per compute unit are not.
uint32_t sqnorm_grid(const cf_ctx *ctx, uint32_t n_chunks)
{
    uint64_t g = n_chunks;
    uint32_t per_cu = ctx->tuning.sqnorm_blocks_per_cu;
    if (per_cu == 0) per_cu = kCappedGridPerCu;
    if (per_cu && per_cu != kOnePerChunk && g > (uint64_t)ctx->num_cu * per_cu) {
        // Every workgroup of the capped grid gets the same number of chunks (or one fewer): with
        // `rounds` passes over the grid, the smallest grid that needs no more passes.
        const uint64_t cap = (uint64_t)ctx->num_cu * per_cu;
        const uint64_t rounds = (n_chunks + cap - 1) / cap;
        g = (n_chunks + rounds - 1) / rounds;
    }
    return (uint32_t)std::max<uint64_t>(g, 1);
}

}  // namespace

extern "C" {

void cf_default_tuning(cf_tuning *out)
{
    if (!out) return;
    out->chunk_bytes = kDefaultChunkBytes;
    out->sqnorm_blocks_per_cu = kDefaultSqnormBlocksPerCu;
    out->reserved0 = 0;
    out->reserved1 = 0;
}

const char *cf_status_string(cf_status status)
{
    switch (status) {
    case CF_OK: return "CF_OK";
    case CF_ERR_NULL: return "CF_ERR_NULL: required pointer is NULL";
    case CF_ERR_SHAPE_MISMATCH: return "CF_ERR_SHAPE_MISMATCH: stages differ in tensor count, numel or dtype";
    case CF_ERR_DTYPE: return "CF_ERR_DTYPE: unknown or unsupported element type";
    case CF_ERR_ALIGN: return "CF_ERR_ALIGN: tensor data not aligned to its element size";
    case CF_ERR_LIMIT: return "CF_ERR_LIMIT: size beyond what the library supports";
    case CF_ERR_HIP: return "CF_ERR_HIP: HIP runtime call failed";
    case CF_ERR_ALIAS: return "CF_ERR_ALIAS: output overlaps an input other than element for element";
    case CF_ERR_CONTEXT: return "CF_ERR_CONTEXT: handles belong to different contexts";
    case CF_ERR_VALUE: return "CF_ERR_VALUE: scalar argument outside its domain";
    default: return "unknown cf_status";
    }
}

uint64_t cf_plan_num_chunks(const cf_tensor *tensors, uint32_t num_tensors, uint32_t chunk_bytes)
{
    if ((num_tensors && !tensors) || !valid_chunk_bytes(chunk_bytes)) return UINT64_MAX;
    uint64_t n = 0;
    for (uint32_t t = 0; t < num_tensors; ++t) {
        if (tensors[t].dtype != CF_F32 && tensors[t].dtype != CF_BF16) return UINT64_MAX;
        n += chunks_of(tensors[t].numel, chunk_bytes / elem_size(tensors[t].dtype));
    }
    return n;
}

cf_status cf_plan_chunks(const cf_tensor *tensors, uint32_t num_tensors, uint32_t chunk_bytes,
                         uint32_t *chunk_tensor, uint64_t *chunk_first, uint32_t *chunk_len, uint64_t cap)
{
    if ((num_tensors && !tensors) || !chunk_tensor || !chunk_first || !chunk_len) return CF_ERR_NULL;
    if (!valid_chunk_bytes(chunk_bytes)) return CF_ERR_LIMIT;
    uint64_t c = 0;
    for (uint32_t t = 0; t < num_tensors; ++t) {
        if (tensors[t].dtype != CF_F32 && tensors[t].dtype != CF_BF16) return CF_ERR_DTYPE;
        const uint64_t chunk_elems = chunk_bytes / elem_size(tensors[t].dtype);
        for (uint64_t first = 0; first < tensors[t].numel; first += chunk_elems) {
            if (c >= cap) return CF_ERR_LIMIT;
            chunk_tensor[c] = t;
            chunk_first[c] = first;
            chunk_len[c] = (uint32_t)std::min<uint64_t>(chunk_elems, tensors[t].numel - first);
            ++c;
        }
    }
    return CF_OK;
}

cf_status cf_check_stage_pair(const cf_tensor *in, uint32_t num_in, const cf_tensor *out, uint32_t num_out)
{
    if ((num_in && !in) || (num_out && !out)) return CF_ERR_NULL;
    try {
        std::vector<HostTensor> vin, vout;
        for (uint32_t t = 0; t < num_in; ++t) {
            cf_status st = check_tensor(in[t]);
            if (st != CF_OK) return st;
            vin.push_back({reinterpret_cast<uint64_t>(in[t].data), in[t].numel, in[t].dtype});
        }
        for (uint32_t t = 0; t < num_out; ++t) {
            cf_status st = check_tensor(out[t]);
            if (st != CF_OK) return st;
            vout.push_back({reinterpret_cast<uint64_t>(out[t].data), out[t].numel, out[t].dtype});
        }
        cf_status st = check_pair(vin, vout);
        if (st != CF_OK) return st;
        return check_self(vout);
    } catch (...) {
        return CF_ERR_LIMIT;   // host memory exhausted
    }
}

uint64_t cf_workspace_bytes(void) { return kCtxWordBytes; }

cf_status cf_ctx_create_in(int device, const cf_tuning *tuning, void *d_workspace, uint64_t workspace_bytes,
                           void *stream, cf_ctx **out)
{
    if (!out) return CF_ERR_NULL;
    *out = nullptr;
    if (!d_workspace) return CF_ERR_NULL;
    if (workspace_bytes < kCtxWordBytes) return CF_ERR_LIMIT;
    if (reinterpret_cast<uint64_t>(d_workspace) % 16 != 0) return CF_ERR_ALIGN;
    cf_tuning t;
    cf_default_tuning(&t);
    if (tuning) {
        if (tuning->chunk_bytes) t.chunk_bytes = tuning->chunk_bytes;
        if (tuning->sqnorm_blocks_per_cu) t.sqnorm_blocks_per_cu = tuning->sqnorm_blocks_per_cu;
    }
    if (!valid_chunk_bytes(t.chunk_bytes) || t.sqnorm_blocks_per_cu > kOnePerChunk) return CF_ERR_LIMIT;

    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return CF_ERR_HIP;
    DeviceGuard guard(device);
    if (!guard.ok()) return CF_ERR_HIP;
    int num_cu = 0;
    if (hipDeviceGetAttribute(&num_cu, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || num_cu <= 0)
        return CF_ERR_HIP;
    cf_ctx *ctx = new (std::nothrow) cf_ctx;
    if (!ctx) return CF_ERR_LIMIT;
    ctx->device = device;
    ctx->num_cu = num_cu;
    ctx->tuning = t;
    for (uint32_t b = t.chunk_bytes / CF_TILE_BYTES; b > 1; b >>= 1) ++ctx->tile_shift;
    ctx->d_words = static_cast<uint32_t *>(d_workspace);
    if (cf_static_scratch_address(device, &ctx->d_static) != hipSuccess) {
        delete ctx;
        return CF_ERR_HIP;
    }
    if (cf_launch_clear_words(ctx->d_words, static_cast<hipStream_t>(stream)) != hipSuccess) {
        delete ctx;
        return CF_ERR_HIP;
    }
    *out = ctx;
    return CF_OK;
}

cf_status cf_ctx_create(int device, const cf_tuning *tuning, cf_ctx **out)
{
    if (!out) return CF_ERR_NULL;
    *out = nullptr;
    if (tuning && ((tuning->chunk_bytes && !valid_chunk_bytes(tuning->chunk_bytes)) || tuning->sqnorm_blocks_per_cu > kOnePerChunk))
        return CF_ERR_LIMIT;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return CF_ERR_HIP;
    DeviceGuard guard(device);
    if (!guard.ok()) return CF_ERR_HIP;
    void *p = nullptr;
    if (hipMalloc(&p, kCtxWordBytes) != hipSuccess) return CF_ERR_HIP;
    cf_status st = cf_ctx_create_in(device, tuning, p, kCtxWordBytes, nullptr, out);
    if (st == CF_OK && hipStreamSynchronize(nullptr) != hipSuccess) {
        delete *out;
        *out = nullptr;
        st = CF_ERR_HIP;
    }
    if (st != CF_OK) {
        (void)hipFree(p);
        return st;
    }
    (*out)->owns_words = true;
    return CF_OK;
}

cf_status cf_ctx_destroy(cf_ctx *ctx)
{
    if (!ctx) return CF_OK;
    if (ctx->live_stages.load() != 0) return CF_ERR_CONTEXT;   // its stages still point at it: nothing is freed
    cf_status st = CF_OK;
    if (ctx->owns_words) {
        DeviceGuard guard(ctx->device);
        if (!guard.ok() || hipFree(ctx->d_words) != hipSuccess) st = CF_ERR_HIP;
    }
    delete ctx;
    return st;
}

uint64_t cf_stage_table_bytes(const cf_ctx *ctx, const cf_tensor *tensors, uint32_t num_tensors)
{
    if (!ctx || (num_tensors && !tensors)) return UINT64_MAX;
    uint64_t n_chunks = 0;
    if (plan_stage(ctx, tensors, num_tensors, &n_chunks) != CF_OK) return UINT64_MAX;
    return table_layout(n_chunks, num_tensors).total;
}

cf_status cf_stage_create_in(cf_ctx *ctx, const cf_tensor *tensors, uint32_t num_tensors, void *d_table,
                             uint64_t table_bytes, void *stream, cf_stage **out)
{
    if (!ctx || !out || (num_tensors && !tensors)) return CF_ERR_NULL;
    *out = nullptr;
    uint64_t n_chunks = 0;
    cf_status st = plan_stage(ctx, tensors, num_tensors, &n_chunks);
    if (st != CF_OK) return st;
    const TableLayout layout = table_layout(n_chunks, num_tensors);
    if (layout.total) {
        if (!d_table) return CF_ERR_NULL;
        if (table_bytes < layout.total) return CF_ERR_LIMIT;
        if (reinterpret_cast<uint64_t>(d_table) % 16 != 0) return CF_ERR_ALIGN;
    }

    cf_stage *stage = new (std::nothrow) cf_stage;
    if (!stage) return CF_ERR_LIMIT;
    stage->ctx = ctx;
    stage->id = g_next_stage_id.fetch_add(1);
    stage->n_chunks = (uint32_t)n_chunks;
    try {
        stage->tensors.reserve(num_tensors);
    } catch (...) {
        delete stage;
        return CF_ERR_LIMIT;   // host memory exhausted
    }
    if (layout.total) {
        char *base = static_cast<char *>(d_table);
        stage->d_table = d_table;
        stage->d_chunks = reinterpret_cast<CfChunk *>(base + layout.chunks_off);
        stage->d_tensor_first = reinterpret_cast<uint32_t *>(base + layout.first_off);
        stage->d_partials = reinterpret_cast<double *>(base + layout.partials_off);
    }
    for (uint32_t t = 0; t < num_tensors; ++t) {
        const cf_tensor &d = tensors[t];
        stage->tensors.push_back({reinterpret_cast<uint64_t>(d.data), d.numel, d.dtype});
        stage->numel += d.numel;
        stage->nbytes += d.numel * elem_size(d.dtype);
    }
    DeviceGuard guard(ctx->device);
    if (!guard.ok() || enqueue_table(ctx, tensors, num_tensors, stage->d_chunks, stage->d_tensor_first, n_chunks,
                                     static_cast<hipStream_t>(stream)) != hipSuccess) {
        delete stage;
        return CF_ERR_HIP;
    }
    ctx->live_stages.fetch_add(1);
    *out = stage;
    return CF_OK;
}

cf_status cf_stage_create(cf_ctx *ctx, const cf_tensor *tensors, uint32_t num_tensors, cf_stage **out)
{
    if (!ctx || !out || (num_tensors && !tensors)) return CF_ERR_NULL;
    *out = nullptr;
    uint64_t n_chunks = 0;
    cf_status st = plan_stage(ctx, tensors, num_tensors, &n_chunks);
    if (st != CF_OK) return st;
    const uint64_t bytes = table_layout(n_chunks, num_tensors).total;
    DeviceGuard guard(ctx->device);
    if (!guard.ok()) return CF_ERR_HIP;
    void *p = nullptr;
    if (bytes && hipMalloc(&p, bytes) != hipSuccess) return CF_ERR_HIP;
    st = cf_stage_create_in(ctx, tensors, num_tensors, p, bytes, nullptr, out);
    if (st == CF_OK && bytes && hipStreamSynchronize(nullptr) != hipSuccess) {
        (void)cf_stage_destroy(*out);
        *out = nullptr;
        st = CF_ERR_HIP;
    }
    if (st != CF_OK) {
        if (p) (void)hipFree(p);
        return st;
    }
    (*out)->owns_table = true;
    return CF_OK;
}

cf_status cf_stage_destroy(cf_stage *stage)
{
    if (!stage) return CF_OK;
    cf_status st = CF_OK;
    forget_stage(stage->ctx, stage->id);
    stage->ctx->live_stages.fetch_sub(1);
    if (stage->owns_table && stage->d_table) {
        DeviceGuard guard(stage->ctx->device);
        if (!guard.ok() || hipFree(stage->d_table) != hipSuccess) st = CF_ERR_HIP;
    }
    delete stage;
    return st;
}

uint32_t cf_stage_num_tensors(const cf_stage *stage) { return stage ? (uint32_t)stage->tensors.size() : 0; }
uint64_t cf_stage_numel(const cf_stage *stage) { return stage ? stage->numel : 0; }
uint64_t cf_stage_nbytes(const cf_stage *stage) { return stage ? stage->nbytes : 0; }
uint32_t cf_stage_num_chunks(const cf_stage *stage) { return stage ? stage->n_chunks : 0; }

cf_status cf_stage_grad_sqnorm(cf_ctx *ctx, const cf_stage *const *grad_stages, uint32_t n_stages,
                               double *d_omega_out, void *stream)
{
    if (!ctx || (n_stages && (!grad_stages || !d_omega_out))) return CF_ERR_NULL;
    for (uint32_t s = 0; s < n_stages; ++s) {
        if (!grad_stages[s]) return CF_ERR_NULL;
        if (grad_stages[s]->ctx != ctx) return CF_ERR_CONTEXT;
    }
    // Every group of stages must fit one launch before anything is launched.
    for (uint32_t base = 0; base < n_stages; base += CF_MAX_SEG) {
        const uint32_t n = std::min<uint32_t>(CF_MAX_SEG, n_stages - base);
        uint64_t total = 0;
        for (uint32_t k = 0; k < n; ++k) total += grad_stages[base + k]->n_chunks;
        if (total >= kMaxChunksPerStage) return CF_ERR_LIMIT;
    }
    DeviceGuard guard(ctx->device);
    if (!guard.ok()) return CF_ERR_HIP;
    for (uint32_t base = 0; base < n_stages; base += CF_MAX_SEG) {
        CfSqnormArgs args;
        std::memset(&args, 0, sizeof args);
        const uint32_t n = std::min<uint32_t>(CF_MAX_SEG, n_stages - base);
        uint64_t total = 0;
        for (uint32_t k = 0; k < n; ++k) {
            const cf_stage *st = grad_stages[base + k];
            args.seg[k].chunks = st->d_chunks;
            args.seg[k].partials = st->d_partials;
            args.seg[k].chunk_begin = (uint32_t)total;
            args.seg[k].n_chunks = st->n_chunks;
            total += st->n_chunks;
        }
        args.n_seg = n;
        args.total_chunks = (uint32_t)total;
        args.omega_out = d_omega_out + base;
        args.words = ctx->d_words;
        const uint32_t grid = sqnorm_grid(ctx, args.total_chunks);
        if (cf_launch_sqnorm(args, grid, static_cast<hipStream_t>(stream)) != hipSuccess) return CF_ERR_HIP;
    }
    return CF_OK;
}

uint64_t cf_static_scratch_bytes(void) { return CF_STATIC_SCRATCH_BYTES; }

cf_status cf_stage_grad_sqnorm_static(cf_ctx *ctx, const cf_tensor *grads, uint32_t num_tensors, double *d_omega_out,
                                      void *stream)
{
    if (!ctx || !d_omega_out || (num_tensors && !grads)) return CF_ERR_NULL;
    uint64_t n_chunks = 0;
    cf_status st = plan_stage(ctx, grads, num_tensors, &n_chunks);
    if (st != CF_OK) return st;
    const TableLayout layout = table_layout(n_chunks, num_tensors);
    if (layout.total > CF_STATIC_SCRATCH_BYTES) return CF_ERR_LIMIT;
    DeviceGuard guard(ctx->device);
    if (!guard.ok()) return CF_ERR_HIP;
    // The tables go where a stage handle would keep them, but inside this device's static array.
    // Nothing in it has to start at zero: the table entries and every partial slot of the stage are
    // written before they are read.
    char *base = static_cast<char *>(ctx->d_static);
    CfChunk *d_chunks = reinterpret_cast<CfChunk *>(base + layout.chunks_off);
    uint32_t *d_tensor_first = reinterpret_cast<uint32_t *>(base + layout.first_off);
    double *d_partials = reinterpret_cast<double *>(base + layout.partials_off);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (enqueue_table(ctx, grads, num_tensors, d_chunks, d_tensor_first, n_chunks, s) != hipSuccess) return CF_ERR_HIP;
    CfSqnormArgs args;
    std::memset(&args, 0, sizeof args);
    args.seg[0].chunks = d_chunks;
    args.seg[0].partials = d_partials;
    args.seg[0].chunk_begin = 0;
    args.seg[0].n_chunks = (uint32_t)n_chunks;
    args.n_seg = 1;
    args.total_chunks = (uint32_t)n_chunks;
    args.omega_out = d_omega_out;
    args.words = ctx->d_words;
    if (cf_launch_sqnorm(args, sqnorm_grid(ctx, args.total_chunks), s) != hipSuccess) return CF_ERR_HIP;
    return CF_OK;
}

cf_status cf_stage_grad_sqnorm_per_tensor(cf_ctx *ctx, const cf_stage *grad_stage, double *d_tensor_sqnorm,
                                          double *d_omega_out, void *stream)
{
    if (!ctx || !grad_stage || !d_omega_out) return CF_ERR_NULL;
    if (!grad_stage->tensors.empty() && !d_tensor_sqnorm) return CF_ERR_NULL;
    const cf_stage *one[1] = {grad_stage};
    cf_status st = cf_stage_grad_sqnorm(ctx, one, 1, d_omega_out, stream);
    if (st != CF_OK) return st;
    if (grad_stage->tensors.empty()) return CF_OK;
    DeviceGuard guard(ctx->device);
    if (!guard.ok()) return CF_ERR_HIP;
    if (cf_launch_sqnorm_tensors(grad_stage->d_partials, grad_stage->d_tensor_first,
                                 (uint32_t)grad_stage->tensors.size(), d_tensor_sqnorm,
                                 static_cast<hipStream_t>(stream)) != hipSuccess)
        return CF_ERR_HIP;
    return CF_OK;
}

namespace {

cf_status recover_impl(cf_ctx *ctx, const cf_stage *prev, const cf_stage *next, const double *d_omega_prev,
                       const double *d_omega_next, double h_omega_prev, double h_omega_next, cf_stage *lost,
                       void *stream)
{
    if (!ctx || !prev || !next || !lost) return CF_ERR_NULL;
    if (prev->ctx != ctx || next->ctx != ctx || lost->ctx != ctx) return CF_ERR_CONTEXT;
    cf_status st = checked_pair(ctx, prev, lost);
    if (st != CF_OK) return st;
    st = checked_pair(ctx, next, lost);
    if (st != CF_OK) return st;
    if (lost->n_chunks == 0) return CF_OK;
    DeviceGuard guard(ctx->device);
    if (!guard.ok()) return CF_ERR_HIP;
    if (cf_launch_blend(prev->d_chunks, next->d_chunks, lost->d_chunks, lost->n_chunks, ctx->tile_shift,
                        d_omega_prev, d_omega_next, h_omega_prev, h_omega_next, ctx->d_words,
                        lost->nbytes >= CF_BLEND_HOLD_MIN_BYTES, static_cast<hipStream_t>(stream)) != hipSuccess)
        return CF_ERR_HIP;
    return CF_OK;
}

}  // namespace

cf_status cf_recover_stage_weighted_avg(cf_ctx *ctx, const cf_stage *prev, const cf_stage *next,
                                        const double *d_omega_prev, const double *d_omega_next,
                                        cf_stage *lost, void *stream)
{
    if (!d_omega_prev || !d_omega_next) return CF_ERR_NULL;
    return recover_impl(ctx, prev, next, d_omega_prev, d_omega_next, 0.0, 0.0, lost, stream);
}

cf_status cf_recover_stage_with_weights(cf_ctx *ctx, const cf_stage *prev, const cf_stage *next,
                                        double omega_prev, double omega_next, cf_stage *lost, void *stream)
{
    return recover_impl(ctx, prev, next, nullptr, nullptr, omega_prev, omega_next, lost, stream);
}

uint64_t cf_adam_scratch_bytes(const cf_stage *grads)
{
    if (!grads) return 0;
    return align_up(((uint64_t)grads->n_chunks << grads->ctx->tile_shift) * sizeof(double));
}

cf_status cf_adam_step_with_sqnorm(cf_ctx *ctx, cf_stage *weights, cf_stage *exp_avg, cf_stage *exp_avg_sq,
                                   const cf_stage *grads, const cf_adam_params *params, void *d_scratch,
                                   uint64_t scratch_bytes, double *d_omega_out, void *stream)
{
    if (!ctx || !weights || !exp_avg || !exp_avg_sq || !grads || !params || !d_omega_out) return CF_ERR_NULL;
    const cf_stage *all[4] = {weights, exp_avg, exp_avg_sq, grads};
    for (const cf_stage *s : all)
        if (s->ctx != ctx) return CF_ERR_CONTEXT;
    const cf_adam_params &a = *params;
    const bool ok = std::isfinite(a.learning_rate) && a.beta1 >= 0.0 && a.beta1 < 1.0 && a.beta2 >= 0.0 &&
                    a.beta2 < 1.0 && std::isfinite(a.epsilon) && a.epsilon >= 0.0 && a.step >= 1;
    if (!ok) return CF_ERR_VALUE;
    for (const cf_stage *s : all)
        for (const HostTensor &t : s->tensors)
            if (t.dtype != CF_F32) return CF_ERR_DTYPE;
    // Every stage written to against every other of the four: congruent, and no byte shared except
    // element for element.
    cf_stage *outs[3] = {weights, exp_avg, exp_avg_sq};
    for (cf_stage *o : outs)
        for (const cf_stage *i : all) {
            if (i == o) continue;
            cf_status st = checked_pair(ctx, i, o);
            if (st != CF_OK) return st;
        }
    const uint64_t need = cf_adam_scratch_bytes(grads);
    if (grads->n_chunks) {
        if (!d_scratch) return CF_ERR_NULL;
        if (scratch_bytes < need) return CF_ERR_LIMIT;
        if (reinterpret_cast<uint64_t>(d_scratch) % 8 != 0) return CF_ERR_ALIGN;
    }
    CfAdamArgs p;
    p.beta1 = a.beta1;
    p.one_minus_beta1 = 1.0 - a.beta1;
    p.beta2 = a.beta2;
    p.one_minus_beta2 = 1.0 - a.beta2;
    p.rcp_correction1 = 1.0 / (1.0 - std::pow(a.beta1, (double)a.step));
    p.rcp_correction2 = 1.0 / (1.0 - std::pow(a.beta2, (double)a.step));
    p.lr = a.learning_rate;
    p.eps = a.epsilon;
    DeviceGuard guard(ctx->device);
    if (!guard.ok()) return CF_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (grads->n_chunks &&
        cf_launch_adam_sqnorm(weights->d_chunks, exp_avg->d_chunks, exp_avg_sq->d_chunks, grads->d_chunks,
                              grads->n_chunks, ctx->tile_shift, p, static_cast<double *>(d_scratch), grads->d_partials,
                              s) != hipSuccess)
        return CF_ERR_HIP;
    CfSqnormArgs args;
    std::memset(&args, 0, sizeof args);
    args.seg[0].chunks = grads->d_chunks;
    args.seg[0].partials = grads->d_partials;
    args.seg[0].n_chunks = grads->n_chunks;
    args.n_seg = 1;
    args.total_chunks = grads->n_chunks;
    args.omega_out = d_omega_out;
    args.words = ctx->d_words;
    if (cf_launch_sqnorm_finalize(args, s) != hipSuccess) return CF_ERR_HIP;
    return CF_OK;
}

double cf_recovered_learning_rate(double learning_rate) { return CF_RECOVERY_LR_FACTOR * learning_rate; }

cf_status cf_plan_recovery(uint32_t num_stages, const uint32_t *lost, uint32_t n_lost, int checkfree_plus,
                           cf_recovery_step *steps)
{
    if (n_lost == 0) return CF_OK;
    if (!lost || !steps) return CF_ERR_NULL;
    for (uint32_t k = 0; k < n_lost; ++k) {
        if (lost[k] >= num_stages) return CF_ERR_LIMIT;
        for (uint32_t j = 0; j < k; ++j)
            if (lost[j] == lost[k]) return CF_ERR_LIMIT;
    }
    const auto alive = [&](uint32_t stage) {
        for (uint32_t k = 0; k < n_lost; ++k)
            if (lost[k] == stage) return false;
        return true;
    };
    const auto step_for = [&](uint32_t i) {
        cf_recovery_step s;
        s.lost = i;
        if (i == 0 || i == num_stages - 1) {
            s.kind = CF_RECOVER_COPY;
            s.prev = s.next = (i == 0) ? 1u : num_stages - 2u;
        } else {
            s.kind = CF_RECOVER_WEIGHTED_AVG;
            s.prev = i - 1u;
            s.next = i + 1u;
        }
        return s;
    };
    // nothing is written unless every lost stage can be rebuilt
    for (uint32_t k = 0; k < n_lost; ++k) {
        if (num_stages < 2) return CF_ERR_LIMIT;   // a single stage has no neighbour at all
        const cf_recovery_step s = step_for(lost[k]);
        if (s.kind == CF_RECOVER_COPY && !checkfree_plus) return CF_ERR_VALUE;
        if (!alive(s.prev) || !alive(s.next)) return CF_ERR_VALUE;
    }
    for (uint32_t k = 0; k < n_lost; ++k) steps[k] = step_for(lost[k]);
    return CF_OK;
}

cf_status cf_plus_stage_order(uint32_t num_stages, uint64_t microbatch, uint32_t *order)
{
    if (!order) return CF_ERR_NULL;
    if (num_stages < 4) return CF_ERR_LIMIT;
    for (uint32_t p = 0; p < num_stages; ++p) order[p] = p;
    if (microbatch & 1u) {
        std::swap(order[0], order[1]);
        std::swap(order[num_stages - 2], order[num_stages - 1]);
    }
    return CF_OK;
}

cf_status cf_copy_stage_range(cf_ctx *ctx, const cf_stage *src, cf_stage *dst, uint32_t first_chunk,
                              uint32_t n_chunks, void *stream)
{
    if (!ctx || !src || !dst) return CF_ERR_NULL;
    if (src->ctx != ctx || dst->ctx != ctx) return CF_ERR_CONTEXT;
    cf_status st = checked_pair(ctx, src, dst);
    if (st != CF_OK) return st;
    if (first_chunk > dst->n_chunks || n_chunks > dst->n_chunks - first_chunk) return CF_ERR_LIMIT;
    if (n_chunks == 0) return CF_OK;
    DeviceGuard guard(ctx->device);
    if (!guard.ok()) return CF_ERR_HIP;
    // The range's size is at most n_chunks whole chunks; whether the stores are held back is a matter of
    // speed only, so the upper bound serves.
    const bool hold = (uint64_t)n_chunks * ctx->tuning.chunk_bytes >= CF_COPY_HOLD_MIN_BYTES;
    if (cf_launch_copy(src->d_chunks, dst->d_chunks, first_chunk, n_chunks, ctx->tile_shift, hold,
                       static_cast<hipStream_t>(stream)) != hipSuccess)
        return CF_ERR_HIP;
    return CF_OK;
}

cf_status cf_copy_stage(cf_ctx *ctx, const cf_stage *src, cf_stage *dst, void *stream)
{
    if (!ctx || !src || !dst) return CF_ERR_NULL;
    return cf_copy_stage_range(ctx, src, dst, 0, dst->n_chunks, stream);
}

cf_status cf_read_flags(cf_ctx *ctx, void *stream, uint32_t *flags, int clear)
{
    if (!ctx || !flags) return CF_ERR_NULL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok()) return CF_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // One kernel behind everything already on `stream` reads the word, and clears it in the same
    // atomic operation when asked to, into a second word that is then brought to the host.
    if (cf_launch_read_flags(ctx->d_words, clear, s) != hipSuccess) return CF_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return CF_ERR_HIP;
    if (hipMemcpy(flags, ctx->d_words + CF_WORD_FLAGS_READ, sizeof(uint32_t), hipMemcpyDeviceToHost) != hipSuccess)
        return CF_ERR_HIP;
    return CF_OK;
}

}  // extern "C"
