// Host side of libpier: the C ABI declared in include/pier.h.  Owns only small
// tables (chunk lists, per-tensor pointer lists, events); every model-sized buffer
// belongs to the caller.
#include "pier_host.h"
#include "pier_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <vector>

using namespace pier;

namespace {
thread_local std::string g_last_error = "";
}

namespace pier {

pier_status fail(pier_status st, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return st;
}

// A pointer handed over as "device memory": must be non-null, aligned to its
// element, and lie with its whole extent inside one allocation of the current GPU.
pier_status check_device_range(const void* ptr, int64_t numel, size_t elem, int device,
                               const char* what, int tensor)
{
    if (numel == 0) return PIER_OK;
    if (!ptr) return fail(PIER_ERR_INVALID_ARG, "%s[%d] is NULL", what, tensor);
    if (reinterpret_cast<uintptr_t>(ptr) % elem)
        return fail(PIER_ERR_ALIGNMENT, "%s[%d] is not aligned to %zu bytes", what, tensor, elem);
    hipPointerAttribute_t at;
    hipError_t e = hipPointerGetAttributes(&at, ptr);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(PIER_ERR_INVALID_ARG, "%s[%d] is not memory known to HIP (%s)", what, tensor,
                    hipGetErrorString(e));
    }
    if (at.type != hipMemoryTypeDevice && at.type != hipMemoryTypeManaged)
        return fail(PIER_ERR_INVALID_ARG, "%s[%d] is not device memory", what, tensor);
    if (at.type == hipMemoryTypeDevice && at.device != device)
        return fail(PIER_ERR_INVALID_ARG, "%s[%d] lives on device %d, context on %d", what, tensor,
                    at.device, device);
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    e = hipMemGetAddressRange(&base, &size, const_cast<void*>(ptr));
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(PIER_ERR_INVALID_ARG, "%s[%d]: cannot query its allocation (%s)", what, tensor,
                    hipGetErrorString(e));
    }
    const char* b = static_cast<const char*>(base);
    const char* q = static_cast<const char*>(ptr);
    if (q < b || q + static_cast<size_t>(numel) * elem > b + size)
        return fail(PIER_ERR_INVALID_ARG, "%s[%d]: %lld elements do not fit its allocation", what,
                    tensor, static_cast<long long>(numel));
    return PIER_OK;
}

}  // namespace pier

// Scratch of the entry point that allocates nothing (pier_inner_adamw_clipped_static): the
// norm pass's record (one ClipState, in the first 256 bytes) followed by its per-workgroup
// partial sums.  One copy per GPU, alive until the process ends, shared by every call on
// that GPU.  In host code this name is only a handle for hipGetSymbolAddress: the device
// address is resolved once per device (scratch_for_current_device) and that pointer is what
// kernels and copies receive.
constexpr int kStaticNormPartials = 16384;
constexpr size_t kScratchHead = 256;
constexpr size_t kScratchBytes = kScratchHead + sizeof(double) * kStaticNormPartials;
static_assert(sizeof(ClipState) <= kScratchHead, "the norm record must fit the head of the scratch");
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

// Device address of `scratch` on each GPU this process has used the library on.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Resolves (once per device, with that device current) where this GPU keeps its copy of
// `scratch`.  Allocates nothing.
pier_status scratch_for_current_device(int device, void** out)
{
    if (device < 0 || device >= kMaxDevices)
        return fail(PIER_ERR_INVALID_ARG, "device %d: the library tracks devices 0..%d", device, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        PIER_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(PIER_ERR_HIP, "hipGetSymbolAddress returned a null address for the scratch array");
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return PIER_OK;
}

// Chunking of one offload piece size: the flat index space cut into pieces, each
// piece owning a contiguous run of chunk-table entries.
struct OffloadPlan {
    int64_t piece_elems = 0;
    std::vector<int64_t> piece_lo;      // n_pieces + 1 flat element bounds
    std::vector<int> chunk_begin;       // n_pieces + 1 indices into the chunk table
    Chunk* d_chunks = nullptr;
    std::vector<hipEvent_t> ev;         // 6 per piece: h2d b/e, kernel b/e, d2h b/e
};

}  // namespace

struct pier_ctx {
    int n_tensors = 0;
    int n_replicas = 0;
    std::vector<int64_t> numel;
    std::vector<int64_t> flat_start;  // n_tensors + 1
    int64_t N = 0;

    // Measured on MI355X at GPT-2 XL size: many small workgroups, each moving one
    // 1024-element tile per stream with streaming (nt) accesses, sustain the highest
    // HBM rate for both kernels; larger chunks or deeper unrolling are 1-5% slower.
    int64_t chunk_elems = 1024;
    LaunchShape shape{1, 0, 1, 0, -1};

    int device = -1;  // set by the first call that touches the GPU
    std::vector<Chunk> h_chunks;
    Chunk* d_chunks = nullptr;
    int n_chunks = 0;

    std::vector<RepPtrs> h_rep;  // n_replicas * n_tensors, replica-major
    RepPtrs* d_rep = nullptr;
    std::vector<char> rep_bound;
    std::vector<char> rep_bf16;
    std::vector<char> rep_shadow;

    int norm_partials = kDefaultNormPartials;  // workgroups (= partial sums) of the norm pass, at most
    double* d_partials = nullptr;  // n_replicas * norm_partials partial sums of the norm pass
    ClipState* d_clip = nullptr;   // one per replica
    std::vector<char> clip_valid;  // 0 = no clipped step yet, 1 = record in d_clip, 2 = record in the static scratch
    void* scratch_ptr = nullptr;   // this GPU's copy of the static scratch (resolved at the first bind)

    std::vector<uint64_t> h_rows;  // n_tensors rows of outer_row_words(n_replicas) words
    uint64_t* d_rows = nullptr;
    bool outer_bound = false;
    pier_loc outer_loc = PIER_LOC_DEVICE;
    float* host_a = nullptr;
    float* host_M = nullptr;

    std::map<size_t, OffloadPlan> plans;
    hipEvent_t offload_done = nullptr;  // end of the previous offload call's copy-back
    bool offload_done_valid = false;
    bool offload_trailing = false;      // compute stream does not wait for the copy-back
};

namespace {

void build_chunks(const pier_ctx* c, int64_t lo, int64_t hi, std::vector<Chunk>& out)
{
    // chunks covering flat elements [lo, hi), never crossing a tensor boundary
    int t = static_cast<int>(std::upper_bound(c->flat_start.begin(), c->flat_start.end(), lo) -
                             c->flat_start.begin()) - 1;
    if (t < 0) t = 0;
    for (; t < c->n_tensors && c->flat_start[t] < hi; ++t) {
        const int64_t b = std::max(lo, c->flat_start[t]) - c->flat_start[t];
        const int64_t e = std::min(hi, c->flat_start[t + 1]) - c->flat_start[t];
        for (int64_t off = b; off < e; off += c->chunk_elems) {
            Chunk ch;
            ch.off = off;
            ch.tensor = t;
            ch.len = static_cast<int32_t>(std::min<int64_t>(c->chunk_elems, e - off));
            out.push_back(ch);
        }
    }
}

void release_tables(pier_ctx* c)
{
    if (c->d_chunks) (void)hipFree(c->d_chunks);
    if (c->d_rep) (void)hipFree(c->d_rep);
    if (c->d_rows) (void)hipFree(c->d_rows);
    if (c->d_partials) (void)hipFree(c->d_partials);
    if (c->d_clip) (void)hipFree(c->d_clip);
    if (c->offload_done) (void)hipEventDestroy(c->offload_done);
    c->d_chunks = nullptr;
    c->d_rep = nullptr;
    c->d_rows = nullptr;
    c->d_partials = nullptr;
    c->d_clip = nullptr;
    c->offload_done = nullptr;
}

pier_status allocate_tables(pier_ctx* c)
{
    c->h_chunks.clear();
    build_chunks(c, 0, c->N, c->h_chunks);
    // a launch has up to four workgroups per chunk and the grid must fit 31 bits
    if (c->h_chunks.size() > static_cast<size_t>(INT32_MAX / 4))
        return fail(PIER_ERR_INVALID_ARG, "too many chunks; raise chunk_elems");
    c->n_chunks = static_cast<int>(c->h_chunks.size());
    if (c->n_chunks > 0) {
        PIER_HIP(hipMalloc(reinterpret_cast<void**>(&c->d_chunks), sizeof(Chunk) * c->n_chunks));
        PIER_HIP(hipMemcpy(c->d_chunks, c->h_chunks.data(), sizeof(Chunk) * c->n_chunks,
                           hipMemcpyHostToDevice));
    }
    const size_t nrep = static_cast<size_t>(c->n_replicas) * c->n_tensors;
    PIER_HIP(hipMalloc(reinterpret_cast<void**>(&c->d_rep), sizeof(RepPtrs) * nrep));
    PIER_HIP(hipMemset(c->d_rep, 0, sizeof(RepPtrs) * nrep));
    PIER_HIP(hipMalloc(reinterpret_cast<void**>(&c->d_rows), sizeof(uint64_t) * c->h_rows.size()));
    PIER_HIP(hipMemcpy(c->d_rows, c->h_rows.data(), sizeof(uint64_t) * c->h_rows.size(),
                       hipMemcpyHostToDevice));
    PIER_HIP(hipMalloc(reinterpret_cast<void**>(&c->d_partials),
                       sizeof(double) * static_cast<size_t>(c->norm_partials) * c->n_replicas));
    PIER_HIP(hipMalloc(reinterpret_cast<void**>(&c->d_clip), sizeof(ClipState) * c->n_replicas));
    PIER_HIP(hipMemset(c->d_clip, 0, sizeof(ClipState) * c->n_replicas));
    PIER_HIP(hipEventCreate(&c->offload_done));
    return PIER_OK;
}

// First GPU contact of a context: remembers the current device and creates the tables
// there (all of them, or none if any allocation fails).
pier_status ensure_device(pier_ctx* c)
{
    int dev = -1;
    PIER_HIP(hipGetDevice(&dev));
    if (c->device >= 0) {
        if (dev != c->device)
            return fail(PIER_ERR_STATE, "context belongs to device %d but device %d is current",
                        c->device, dev);
        return PIER_OK;
    }
    pier_status st = scratch_for_current_device(dev, &c->scratch_ptr);
    if (st != PIER_OK) return st;
    st = allocate_tables(c);
    if (st != PIER_OK) {
        release_tables(c);
        return st;
    }
    c->device = dev;
    return PIER_OK;
}

pier_status check_outer_hp(const pier_outer_hp* hp)
{
    if (!hp) return fail(PIER_ERR_INVALID_ARG, "hp is NULL");
    if (hp->phase != PIER_PHASE_WARMUP && hp->phase != PIER_PHASE_PIER)
        return fail(PIER_ERR_INVALID_ARG, "hp->phase is neither WARMUP nor PIER");
    if (!std::isfinite(hp->mu) || !std::isfinite(hp->outer_lr))
        return fail(PIER_ERR_INVALID_ARG, "hp->mu / hp->outer_lr is not finite");
    return PIER_OK;
}

pier_status check_all_bound(const pier_ctx* c)
{
    for (int r = 0; r < c->n_replicas; ++r)
        if (!c->rep_bound[r]) return fail(PIER_ERR_STATE, "replica %d is not bound", r);
    return PIER_OK;
}

// Word 3 of every outer-table row: alignment of the tensor's theta and working-copy pointers
// over all replicas (the kernel for arbitrary group counts picks its vector path from it).
void refresh_row_flags(pier_ctx* c)
{
    const size_t rw = outer_row_words(c->n_replicas);
    for (int i = 0; i < c->n_tensors; ++i) {
        uint64_t th = 0, wb = 0;
        for (int r = 0; r < c->n_replicas; ++r) {
            th |= c->h_rows[rw * i + kOuterRowHead + r];
            wb |= c->h_rows[rw * i + kOuterRowHead + c->n_replicas + r];
        }
        c->h_rows[rw * i + 3] = ((th & 15u) == 0 ? 1u : 0u) | ((wb & 7u) == 0 ? 2u : 0u);
    }
}

void free_plan(OffloadPlan& p)
{
    if (p.d_chunks) (void)hipFree(p.d_chunks);
    for (hipEvent_t e : p.ev) (void)hipEventDestroy(e);
    p.ev.clear();
    p.d_chunks = nullptr;
}

}  // namespace

extern "C" {

int pier_abi_version(void) { return PIER_ABI_VERSION; }

const char* pier_last_error(void) { return g_last_error.c_str(); }

const char* pier_status_string(pier_status s)
{
    switch (s) {
    case PIER_OK: return "PIER_OK";
    case PIER_ERR_INVALID_ARG: return "PIER_ERR_INVALID_ARG";
    case PIER_ERR_ALIGNMENT: return "PIER_ERR_ALIGNMENT";
    case PIER_ERR_STATE: return "PIER_ERR_STATE";
    case PIER_ERR_OOM: return "PIER_ERR_OOM";
    case PIER_ERR_HIP: return "PIER_ERR_HIP";
    }
    return "PIER_ERR_UNKNOWN";
}

pier_status pier_ctx_create(pier_ctx** out, int n_tensors, const int64_t* numel, int n_replicas)
{
    if (!out) return fail(PIER_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (n_tensors < 1) return fail(PIER_ERR_INVALID_ARG, "n_tensors = %d, need >= 1", n_tensors);
    if (!numel) return fail(PIER_ERR_INVALID_ARG, "numel is NULL");
    if (n_replicas < 1 || n_replicas > PIER_MAX_REPLICAS)
        return fail(PIER_ERR_INVALID_ARG, "n_replicas = %d, need 1..%d", n_replicas,
                    PIER_MAX_REPLICAS);
    pier_ctx* c = new (std::nothrow) pier_ctx;
    if (!c) return fail(PIER_ERR_OOM, "out of host memory");
    try {
        c->n_tensors = n_tensors;
        c->n_replicas = n_replicas;
        c->numel.assign(numel, numel + n_tensors);
        c->flat_start.assign(n_tensors + 1, 0);
        for (int i = 0; i < n_tensors; ++i) {
            if (numel[i] < 0) {
                delete c;
                return fail(PIER_ERR_INVALID_ARG, "numel[%d] = %lld is negative", i,
                            static_cast<long long>(numel[i]));
            }
            if (numel[i] > INT64_MAX / 8 - c->flat_start[i]) {
                delete c;
                return fail(PIER_ERR_INVALID_ARG, "total element count overflows");
            }
            c->flat_start[i + 1] = c->flat_start[i] + numel[i];
        }
        c->N = c->flat_start[n_tensors];
        c->h_rep.assign(static_cast<size_t>(n_replicas) * n_tensors, RepPtrs{});
        c->rep_bound.assign(n_replicas, 0);
        c->rep_bf16.assign(n_replicas, 0);
        c->rep_shadow.assign(n_replicas, 0);
        c->clip_valid.assign(n_replicas, 0);
        const size_t rw = outer_row_words(n_replicas);
        c->h_rows.assign(rw * n_tensors, 0);
        for (int i = 0; i < n_tensors; ++i) c->h_rows[rw * i + 2] = static_cast<uint64_t>(c->flat_start[i]);
    } catch (const std::bad_alloc&) {
        delete c;
        return fail(PIER_ERR_OOM, "out of host memory");
    }
    *out = c;
    return PIER_OK;
}

pier_status pier_ctx_destroy(pier_ctx* c)
{
    if (!c) return fail(PIER_ERR_INVALID_ARG, "ctx is NULL");
    if (c->device >= 0) {
        release_tables(c);
        for (auto& kv : c->plans) free_plan(kv.second);
    }
    delete c;
    return PIER_OK;
}

int64_t pier_ctx_numel(const pier_ctx* c) { return c ? c->N : -1; }

pier_status pier_ctx_set_launch(pier_ctx* c, int64_t chunk_elems, int unroll, int max_grid,
                                int nontemporal)
{
    if (!c) return fail(PIER_ERR_INVALID_ARG, "ctx is NULL");
    if (c->device >= 0) return fail(PIER_ERR_STATE, "launch shape must be set before the first bind");
    if (chunk_elems != 0) {
        if (chunk_elems < 1024 || chunk_elems % 1024 || chunk_elems > (1 << 26))
            return fail(PIER_ERR_INVALID_ARG, "chunk_elems = %lld: need a multiple of 1024 in [1024, 2^26]",
                        static_cast<long long>(chunk_elems));
    }
    if (unroll != 0 && unroll != 1 && unroll != 2 && unroll != 4)
        return fail(PIER_ERR_INVALID_ARG, "unroll = %d: need 1, 2 or 4", unroll);
    if (max_grid < 0) return fail(PIER_ERR_INVALID_ARG, "max_grid is negative");
    if (nontemporal < -1 || nontemporal > 1)
        return fail(PIER_ERR_INVALID_ARG, "nontemporal = %d: need 0, 1 or -1", nontemporal);
    if (chunk_elems) c->chunk_elems = chunk_elems;
    if (unroll) c->shape.unroll = unroll;
    c->shape.max_grid = max_grid;
    if (nontemporal >= 0) c->shape.nontemporal = nontemporal;
    return PIER_OK;
}

pier_status pier_ctx_set_norm_fold(pier_ctx* c, int n_partials)
{
    if (!c) return fail(PIER_ERR_INVALID_ARG, "ctx is NULL");
    if (c->device >= 0) return fail(PIER_ERR_STATE, "the norm fold width must be set before the first bind");
    if (n_partials == 0) n_partials = kDefaultNormPartials;
    if (n_partials < 1 || n_partials > (1 << 20))
        return fail(PIER_ERR_INVALID_ARG, "n_partials = %d: need 1 .. 2^20, or 0 for the default", n_partials);
    c->norm_partials = n_partials;
    return PIER_OK;
}

pier_status pier_ctx_set_occupancy(pier_ctx* c, int wg_threads, int lds_bytes)
{
    if (!c) return fail(PIER_ERR_INVALID_ARG, "ctx is NULL");
    if (wg_threads != 0 && wg_threads != 64 && wg_threads != kBlock)
        return fail(PIER_ERR_INVALID_ARG, "wg_threads = %d: need 64, %d or 0", wg_threads, kBlock);
    if (lds_bytes < -1 || lds_bytes > 65536)
        return fail(PIER_ERR_INVALID_ARG, "lds_bytes = %d: need 0 .. 65536, or -1", lds_bytes);
    c->shape.wg_threads = wg_threads;
    c->shape.lds_bytes = lds_bytes;
    return PIER_OK;
}

pier_status pier_bind_replica(pier_ctx* c, int replica, float* const* p, float* const* m,
                              float* const* v, const void* const* grad, int grad_is_bf16)
{
    if (!c) return fail(PIER_ERR_INVALID_ARG, "ctx is NULL");
    if (replica < 0 || replica >= c->n_replicas)
        return fail(PIER_ERR_INVALID_ARG, "replica = %d, context has %d", replica, c->n_replicas);
    if (!p || !m || !v || !grad) return fail(PIER_ERR_INVALID_ARG, "a pointer list is NULL");
    pier_status st = ensure_device(c);
    if (st != PIER_OK) return st;
    const size_t gelem = grad_is_bf16 ? 2 : 4;
    for (int i = 0; i < c->n_tensors; ++i) {
        const int64_t n = c->numel[i];
        if ((st = check_device_range(p[i], n, 4, c->device, "p", i)) != PIER_OK) return st;
        if ((st = check_device_range(m[i], n, 4, c->device, "m", i)) != PIER_OK) return st;
        if ((st = check_device_range(v[i], n, 4, c->device, "v", i)) != PIER_OK) return st;
        if ((st = check_device_range(grad[i], n, gelem, c->device, "grad", i)) != PIER_OK) return st;
    }
    RepPtrs* row = c->h_rep.data() + static_cast<size_t>(replica) * c->n_tensors;
    for (int i = 0; i < c->n_tensors; ++i) {
        row[i].p = p[i];
        row[i].m = m[i];
        row[i].v = v[i];
        row[i].g = grad[i];
    }
    PIER_HIP(hipMemcpy(c->d_rep + static_cast<size_t>(replica) * c->n_tensors, row,
                       sizeof(RepPtrs) * c->n_tensors, hipMemcpyHostToDevice));
    const size_t rw = outer_row_words(c->n_replicas);
    for (int i = 0; i < c->n_tensors; ++i)
        c->h_rows[rw * i + kOuterRowHead + replica] = reinterpret_cast<uint64_t>(p[i]);
    refresh_row_flags(c);
    PIER_HIP(hipMemcpy(c->d_rows, c->h_rows.data(), sizeof(uint64_t) * c->h_rows.size(),
                       hipMemcpyHostToDevice));
    c->rep_bound[replica] = 1;
    c->rep_bf16[replica] = grad_is_bf16 ? 1 : 0;
    return PIER_OK;
}

pier_status pier_bind_shadow(pier_ctx* c, int replica, uint16_t* const* w_bf16)
{
    if (!c) return fail(PIER_ERR_INVALID_ARG, "ctx is NULL");
    if (replica < 0 || replica >= c->n_replicas)
        return fail(PIER_ERR_INVALID_ARG, "replica = %d, context has %d", replica, c->n_replicas);
    pier_status st = ensure_device(c);
    if (st != PIER_OK) return st;
    if (w_bf16)
        for (int i = 0; i < c->n_tensors; ++i)
            if ((st = check_device_range(w_bf16[i], c->numel[i], 2, c->device, "w_bf16", i)) != PIER_OK) return st;
    RepPtrs* row = c->h_rep.data() + static_cast<size_t>(replica) * c->n_tensors;
    const size_t rw = outer_row_words(c->n_replicas);
    for (int i = 0; i < c->n_tensors; ++i) {
        row[i].w = w_bf16 ? w_bf16[i] : nullptr;
        c->h_rows[rw * i + kOuterRowHead + c->n_replicas + replica] = reinterpret_cast<uint64_t>(row[i].w);
    }
    refresh_row_flags(c);
    PIER_HIP(hipMemcpy(c->d_rep + static_cast<size_t>(replica) * c->n_tensors, row,
                       sizeof(RepPtrs) * c->n_tensors, hipMemcpyHostToDevice));
    PIER_HIP(hipMemcpy(c->d_rows, c->h_rows.data(), sizeof(uint64_t) * c->h_rows.size(),
                       hipMemcpyHostToDevice));
    c->rep_shadow[replica] = w_bf16 ? 1 : 0;
    return PIER_OK;
}

// The fused outer step writes the working copies of all replicas or of none.
static pier_status outer_shadow_mode(const pier_ctx* c, bool* shadow)
{
    int n = 0;
    for (int r = 0; r < c->n_replicas; ++r) n += c->rep_shadow[r] ? 1 : 0;
    if (n != 0 && n != c->n_replicas)
        return fail(PIER_ERR_STATE, "bfloat16 working copies are bound for %d of %d replicas; bind all or none",
                    n, c->n_replicas);
    *shadow = n != 0;
    return PIER_OK;
}

pier_status pier_bind_outer(pier_ctx* c, pier_loc loc, float* const* anchor,
                            float* const* momentum)
{
    if (!c) return fail(PIER_ERR_INVALID_ARG, "ctx is NULL");
    if (loc != PIER_LOC_DEVICE && loc != PIER_LOC_HOST_PINNED)
        return fail(PIER_ERR_INVALID_ARG, "loc is neither DEVICE nor HOST_PINNED");
    if (!anchor || !momentum) return fail(PIER_ERR_INVALID_ARG, "a pointer list is NULL");
    pier_status st = ensure_device(c);
    if (st != PIER_OK) return st;
    if (loc == PIER_LOC_DEVICE) {
        for (int i = 0; i < c->n_tensors; ++i) {
            if ((st = check_device_range(anchor[i], c->numel[i], 4, c->device, "anchor", i)) != PIER_OK) return st;
            if ((st = check_device_range(momentum[i], c->numel[i], 4, c->device, "momentum", i)) != PIER_OK) return st;
        }
        const size_t rw = outer_row_words(c->n_replicas);
        for (int i = 0; i < c->n_tensors; ++i) {
            c->h_rows[rw * i + 0] = reinterpret_cast<uint64_t>(anchor[i]);
            c->h_rows[rw * i + 1] = reinterpret_cast<uint64_t>(momentum[i]);
        }
        PIER_HIP(hipMemcpy(c->d_rows, c->h_rows.data(), sizeof(uint64_t) * c->h_rows.size(),
                           hipMemcpyHostToDevice));
        c->host_a = c->host_M = nullptr;
    } else {
        float* arr[2] = {anchor[0], momentum[0]};
        const char* names[2] = {"anchor", "momentum"};
        for (int k = 0; k < 2; ++k) {
            if (c->N == 0) break;
            if (!arr[k]) return fail(PIER_ERR_INVALID_ARG, "%s[0] is NULL", names[k]);
            if (reinterpret_cast<uintptr_t>(arr[k]) % 4)
                return fail(PIER_ERR_ALIGNMENT, "%s[0] is not aligned to 4 bytes", names[k]);
            hipPointerAttribute_t at;
            hipError_t e = hipPointerGetAttributes(&at, arr[k]);
            if (e != hipSuccess || at.type != hipMemoryTypeHost) {
                (void)hipGetLastError();
                return fail(PIER_ERR_INVALID_ARG, "%s[0] is not pinned host memory", names[k]);
            }
        }
        c->host_a = arr[0];
        c->host_M = arr[1];
    }
    c->outer_loc = loc;
    c->outer_bound = true;
    return PIER_OK;
}

// Where the norm pass of a clipped step keeps its partial sums and its record.
enum ClipMode { kNoClip = 0, kClipCtx = 1, kClipStatic = 2 };

// Every check of an inner step; launches nothing.
static pier_status inner_adamw_validate(pier_ctx* c, int replica, const pier_adamw_hp* hp, ClipMode clip,
                                        float max_norm)
{
    if (!c) return fail(PIER_ERR_INVALID_ARG, "ctx is NULL");
    if (!hp) return fail(PIER_ERR_INVALID_ARG, "hp is NULL");
    if (replica < 0 || replica >= c->n_replicas)
        return fail(PIER_ERR_INVALID_ARG, "replica = %d, context has %d", replica, c->n_replicas);
    if (!c->rep_bound[replica]) return fail(PIER_ERR_STATE, "replica %d is not bound", replica);
    if (hp->step < 1) return fail(PIER_ERR_INVALID_ARG, "step = %lld, need >= 1", static_cast<long long>(hp->step));
    if (!(hp->beta1 >= 0.0f && hp->beta1 < 1.0f) || !(hp->beta2 >= 0.0f && hp->beta2 < 1.0f))
        return fail(PIER_ERR_INVALID_ARG, "betas must lie in [0, 1)");
    if (!std::isfinite(hp->lr) || !std::isfinite(hp->eps) || !std::isfinite(hp->weight_decay) ||
        !std::isfinite(hp->grad_scale) || hp->eps < 0.0f)
        return fail(PIER_ERR_INVALID_ARG, "lr / eps / weight_decay / grad_scale not finite, or eps < 0");
    if (clip != kNoClip && !(max_norm > 0.0f && std::isfinite(max_norm)))
        return fail(PIER_ERR_INVALID_ARG, "max_norm = %g, need a positive finite value", static_cast<double>(max_norm));
    pier_status st = ensure_device(c);
    if (st != PIER_OK) return st;
    if (clip == kClipStatic) {
        const int n_partials = std::min(c->n_chunks, c->norm_partials);
        const size_t need = kScratchHead + sizeof(double) * static_cast<size_t>(n_partials);
        if (need > kScratchBytes)
            return fail(PIER_ERR_INVALID_ARG,
                        "the norm pass of this context folds %d partial sums and needs %zu bytes of scratch; "
                        "the static scratch holds %zu (at most %d partial sums)",
                        n_partials, need, kScratchBytes, kStaticNormPartials);
    }
    return PIER_OK;
}

// The launches of a validated inner step.
static pier_status inner_adamw_enqueue(pier_ctx* c, int replica, const pier_adamw_hp* hp, ClipMode clip,
                                       float max_norm, void* hip_stream)
{
    AdamwScalars s;
    s.lr = hp->lr;
    s.beta1 = hp->beta1;
    s.beta2 = hp->beta2;
    s.om1 = 1.0f - hp->beta1;
    s.om2 = 1.0f - hp->beta2;
    s.eps = hp->eps;
    s.wd = hp->weight_decay;
    // bias corrections 1 - beta^t: formed in double, applied in fp32
    s.bc1 = static_cast<float>(1.0 - std::pow(static_cast<double>(hp->beta1), static_cast<double>(hp->step)));
    s.bc2 = static_cast<float>(1.0 - std::pow(static_cast<double>(hp->beta2), static_cast<double>(hp->step)));
    s.grad_scale = hp->grad_scale;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const RepPtrs* tab = c->d_rep + static_cast<size_t>(replica) * c->n_tensors;
    const ClipState* cs = nullptr;
    if (clip != kNoClip) {
        // every partial sum the fold reads and the whole record are rewritten by this call, so
        // nothing in either buffer has to start at zero
        const int n_partials = std::min(c->n_chunks, c->norm_partials);
        double* partials;
        ClipState* record;
        if (clip == kClipStatic) {
            record = static_cast<ClipState*>(c->scratch_ptr);
            partials = reinterpret_cast<double*>(static_cast<unsigned char*>(c->scratch_ptr) + kScratchHead);
        } else {
            record = c->d_clip + replica;
            partials = c->d_partials + static_cast<size_t>(replica) * c->norm_partials;
        }
        PIER_HIP(launch_grad_norm(c->d_chunks, c->n_chunks, tab, c->rep_bf16[replica] != 0, partials,
                                  n_partials, max_norm, record, stream));
        c->clip_valid[replica] = static_cast<char>(clip);
        cs = record;
    }
    PIER_HIP(launch_adamw(c->d_chunks, c->n_chunks, tab, c->rep_bf16[replica] != 0,
                          c->rep_shadow[replica] != 0, s, cs, c->shape, stream));
    return PIER_OK;
}

static pier_status inner_adamw_impl(pier_ctx* c, int replica, const pier_adamw_hp* hp, ClipMode clip,
                                    float max_norm, void* hip_stream)
{
    const pier_status st = inner_adamw_validate(c, replica, hp, clip, max_norm);
    if (st != PIER_OK) return st;
    return inner_adamw_enqueue(c, replica, hp, clip, max_norm, hip_stream);
}

pier_status pier_inner_adamw(pier_ctx* c, int replica, const pier_adamw_hp* hp, void* hip_stream)
{
    return inner_adamw_impl(c, replica, hp, kNoClip, 0.0f, hip_stream);
}

pier_status pier_inner_adamw_clipped(pier_ctx* c, int replica, const pier_adamw_hp* hp, float max_norm,
                                     void* hip_stream)
{
    return inner_adamw_impl(c, replica, hp, kClipCtx, max_norm, hip_stream);
}

pier_status pier_inner_adamw_clipped_static(pier_ctx* c, int replica, const pier_adamw_hp* hp, float max_norm,
                                            void* hip_stream)
{
    return inner_adamw_impl(c, replica, hp, kClipStatic, max_norm, hip_stream);
}

pier_status pier_grad_norm_last(pier_ctx* c, int replica, double* norm_out, float* coef_out,
                                void* hip_stream)
{
    if (!c) return fail(PIER_ERR_INVALID_ARG, "ctx is NULL");
    if (replica < 0 || replica >= c->n_replicas)
        return fail(PIER_ERR_INVALID_ARG, "replica = %d, context has %d", replica, c->n_replicas);
    if (c->device < 0 || !c->clip_valid[replica])
        return fail(PIER_ERR_STATE, "replica %d has not run a clipped step", replica);
    pier_status st = ensure_device(c);
    if (st != PIER_OK) return st;
    ClipState h;
    const ClipState* src = c->clip_valid[replica] == kClipStatic ? static_cast<const ClipState*>(c->scratch_ptr)
                                                                 : c->d_clip + replica;
    PIER_HIP(hipMemcpyAsync(&h, src, sizeof h, hipMemcpyDeviceToHost, static_cast<hipStream_t>(hip_stream)));
    PIER_HIP(hipStreamSynchronize(static_cast<hipStream_t>(hip_stream)));
    if (norm_out) *norm_out = h.norm;
    if (coef_out) *coef_out = h.coef;
    return PIER_OK;
}

// Every check of the resident outer step; launches nothing.
static pier_status outer_step_validate(pier_ctx* c, const pier_outer_hp* hp, bool* shadow)
{
    if (!c) return fail(PIER_ERR_INVALID_ARG, "ctx is NULL");
    pier_status st = check_outer_hp(hp);
    if (st != PIER_OK) return st;
    if ((st = check_all_bound(c)) != PIER_OK) return st;
    if (!c->outer_bound || c->outer_loc != PIER_LOC_DEVICE)
        return fail(PIER_ERR_STATE, "anchor and momentum are not bound as device tensors");
    if ((st = ensure_device(c)) != PIER_OK) return st;
    return outer_shadow_mode(c, shadow);
}

pier_status pier_outer_step(pier_ctx* c, const pier_outer_hp* hp, void* hip_stream)
{
    bool shadow = false;
    const pier_status st = outer_step_validate(c, hp, &shadow);
    if (st != PIER_OK) return st;
    PIER_HIP(launch_outer(c->d_chunks, c->n_chunks, c->d_rows, c->n_replicas, nullptr, nullptr, 0,
                          hp->mu, hp->outer_lr, hp->phase == PIER_PHASE_PIER, shadow, c->shape,
                          static_cast<hipStream_t>(hip_stream)));
    return PIER_OK;
}

pier_status pier_offload_workspace_bytes(const pier_ctx* c, size_t chunk_bytes, size_t* out)
{
    if (!c || !out) return fail(PIER_ERR_INVALID_ARG, "ctx or out is NULL");
    if (chunk_bytes < 16 || chunk_bytes % 16)
        return fail(PIER_ERR_INVALID_ARG, "chunk_bytes must be a positive multiple of 16");
    const size_t total = static_cast<size_t>(c->N) * 4;
    const size_t piece = std::min(chunk_bytes, std::max<size_t>(16, (total + 15) / 16 * 16));
    const size_t n_pieces = (total + piece - 1) / piece;
    *out = 2 * piece * std::max<size_t>(1, std::min<size_t>(3, n_pieces));
    return PIER_OK;
}

pier_status pier_ctx_set_offload_writeback(pier_ctx* c, int trailing)
{
    if (!c) return fail(PIER_ERR_INVALID_ARG, "ctx is NULL");
    if (trailing != 0 && trailing != 1) return fail(PIER_ERR_INVALID_ARG, "trailing = %d: need 0 or 1", trailing);
    c->offload_trailing = trailing != 0;
    return PIER_OK;
}

// What a validated offload call works with.
struct OffloadSetup {
    OffloadPlan* plan = nullptr;
    size_t piece_bytes = 0;
    size_t total = 0;
    int n_pieces = 0;
    int n_slots = 0;
    bool shadow = false;
};

// Every check of the offloaded outer step, and the chunking of this piece size (built and
// uploaded the first time it is asked for: table memory of the library, no caller buffer).
// Enqueues nothing on the caller's streams.  N == 0 leaves `out->plan` null.
static pier_status offload_validate(pier_ctx* c, const pier_outer_hp* hp, size_t chunk_bytes, void* workspace,
                                    size_t workspace_bytes, OffloadSetup* out)
{
    if (!c) return fail(PIER_ERR_INVALID_ARG, "ctx is NULL");
    pier_status st = check_outer_hp(hp);
    if (st != PIER_OK) return st;
    if ((st = check_all_bound(c)) != PIER_OK) return st;
    if (!c->outer_bound || c->outer_loc != PIER_LOC_HOST_PINNED)
        return fail(PIER_ERR_STATE, "anchor and momentum are not bound as pinned host arrays");
    if (chunk_bytes < 16 || chunk_bytes % 16)
        return fail(PIER_ERR_INVALID_ARG, "chunk_bytes must be a positive multiple of 16");
    if ((st = ensure_device(c)) != PIER_OK) return st;
    if ((st = outer_shadow_mode(c, &out->shadow)) != PIER_OK) return st;
    if (c->N == 0) return PIER_OK;

    const size_t total = static_cast<size_t>(c->N) * 4;
    const size_t piece_bytes = std::min(chunk_bytes, (total + 15) / 16 * 16);
    const int64_t piece_elems = static_cast<int64_t>(piece_bytes / 4);
    const int n_pieces = static_cast<int>((c->N + piece_elems - 1) / piece_elems);
    const int n_slots = static_cast<int>(std::min<size_t>(std::min<size_t>(64, n_pieces),
                                                          workspace_bytes / (2 * piece_bytes)));
    if (n_slots < 1)
        return fail(PIER_ERR_INVALID_ARG, "workspace of %zu bytes holds no staging slot of 2 x %zu bytes",
                    workspace_bytes, piece_bytes);
    if ((st = check_device_range(workspace, static_cast<int64_t>(2 * piece_bytes) * n_slots, 1,
                                 c->device, "workspace", 0)) != PIER_OK) return st;
    if (reinterpret_cast<uintptr_t>(workspace) % 16)
        return fail(PIER_ERR_ALIGNMENT, "workspace is not aligned to 16 bytes");

    OffloadPlan& plan = c->plans[piece_bytes];
    if (plan.piece_elems == 0) {
        std::vector<Chunk> chunks;
        plan.piece_lo.clear();
        plan.chunk_begin.clear();
        for (int k = 0; k < n_pieces; ++k) {
            const int64_t lo = k * piece_elems, hi = std::min<int64_t>(c->N, lo + piece_elems);
            plan.piece_lo.push_back(lo);
            plan.chunk_begin.push_back(static_cast<int>(chunks.size()));
            build_chunks(c, lo, hi, chunks);
        }
        plan.piece_lo.push_back(c->N);
        plan.chunk_begin.push_back(static_cast<int>(chunks.size()));
        hipError_t e = hipMalloc(reinterpret_cast<void**>(&plan.d_chunks), sizeof(Chunk) * chunks.size());
        if (e == hipSuccess)
            e = hipMemcpy(plan.d_chunks, chunks.data(), sizeof(Chunk) * chunks.size(), hipMemcpyHostToDevice);
        for (int i = 0; e == hipSuccess && i < 6 * n_pieces; ++i) {
            hipEvent_t ev = nullptr;
            e = hipEventCreate(&ev);
            if (e == hipSuccess) plan.ev.push_back(ev);
        }
        if (e != hipSuccess) {
            free_plan(plan);
            c->plans.erase(piece_bytes);
            return fail(e == hipErrorOutOfMemory ? PIER_ERR_OOM : PIER_ERR_HIP, "building the offload plan: %s",
                        hipGetErrorString(e));
        }
        plan.piece_elems = piece_elems;
    }
    out->plan = &plan;
    out->piece_bytes = piece_bytes;
    out->total = total;
    out->n_pieces = n_pieces;
    out->n_slots = n_slots;
    return PIER_OK;
}

// The copies and launches of a validated offload call.
static pier_status offload_enqueue(pier_ctx* c, const pier_outer_hp* hp, const OffloadSetup& S, void* workspace,
                                   void* compute_stream, void* h2d_stream, void* d2h_stream,
                                   pier_offload_stats* stats)
{
    if (stats) std::memset(stats, 0, sizeof *stats);
    if (!S.plan) return PIER_OK;      // empty model
    OffloadPlan& plan = *S.plan;
    const size_t piece_bytes = S.piece_bytes, total = S.total;
    const int n_pieces = S.n_pieces, n_slots = S.n_slots;
    const bool shadow = S.shadow;

    hipStream_t sc = static_cast<hipStream_t>(compute_stream);
    hipStream_t sin = static_cast<hipStream_t>(h2d_stream);
    hipStream_t sout = static_cast<hipStream_t>(d2h_stream);
    char* ws = static_cast<char*>(workspace);
    auto EV = [&](int k, int which) { return plan.ev[static_cast<size_t>(k) * 6 + which]; };
    enum { H2D_B, H2D_E, KER_B, KER_E, D2H_B, D2H_E };

    // the host arrays and the staging slots may still be in use by the previous call
    if (c->offload_done_valid) PIER_HIP(hipStreamWaitEvent(sin, c->offload_done, 0));

    for (int k = 0; k < n_pieces; ++k) {
        const int slot = k % n_slots;
        float* sa = reinterpret_cast<float*>(ws + static_cast<size_t>(slot) * 2 * piece_bytes);
        float* sM = reinterpret_cast<float*>(ws + static_cast<size_t>(slot) * 2 * piece_bytes + piece_bytes);
        const int64_t lo = plan.piece_lo[k], hi = plan.piece_lo[k + 1];
        const size_t bytes = static_cast<size_t>(hi - lo) * 4;

        // stage 1: reload the previous model and the momentum of this piece
        if (k >= n_slots) PIER_HIP(hipStreamWaitEvent(sin, EV(k - n_slots, D2H_E), 0));
        PIER_HIP(hipEventRecord(EV(k, H2D_B), sin));
        PIER_HIP(hipMemcpyAsync(sa, c->host_a + lo, bytes, hipMemcpyHostToDevice, sin));
        PIER_HIP(hipMemcpyAsync(sM, c->host_M + lo, bytes, hipMemcpyHostToDevice, sin));
        PIER_HIP(hipEventRecord(EV(k, H2D_E), sin));

        // stage 2: the outer step on this piece
        PIER_HIP(hipStreamWaitEvent(sc, EV(k, H2D_E), 0));
        PIER_HIP(hipEventRecord(EV(k, KER_B), sc));
        PIER_HIP(launch_outer(plan.d_chunks + plan.chunk_begin[k],
                              plan.chunk_begin[k + 1] - plan.chunk_begin[k], c->d_rows, c->n_replicas,
                              sa, sM, lo, hp->mu, hp->outer_lr, hp->phase == PIER_PHASE_PIER, shadow,
                              c->shape, sc));
        PIER_HIP(hipEventRecord(EV(k, KER_E), sc));

        // stage 3: offload the new model and momentum of this piece
        PIER_HIP(hipStreamWaitEvent(sout, EV(k, KER_E), 0));
        PIER_HIP(hipEventRecord(EV(k, D2H_B), sout));
        PIER_HIP(hipMemcpyAsync(c->host_a + lo, sa, bytes, hipMemcpyDeviceToHost, sout));
        PIER_HIP(hipMemcpyAsync(c->host_M + lo, sM, bytes, hipMemcpyDeviceToHost, sout));
        PIER_HIP(hipEventRecord(EV(k, D2H_E), sout));
    }
    PIER_HIP(hipEventRecord(c->offload_done, sout));
    c->offload_done_valid = true;
    if (!c->offload_trailing) PIER_HIP(hipStreamWaitEvent(sc, c->offload_done, 0));

    if (stats) {
        PIER_HIP(hipEventSynchronize(c->offload_done));
        stats->n_pieces = n_pieces;
        stats->n_slots = n_slots;
        stats->h2d_bytes = stats->d2h_bytes = 2.0 * static_cast<double>(total);
        for (int k = 0; k < n_pieces; ++k) {
            float ms = 0.f;
            PIER_HIP(hipEventElapsedTime(&ms, EV(k, H2D_B), EV(k, H2D_E)));
            stats->h2d_ms += ms;
            PIER_HIP(hipEventElapsedTime(&ms, EV(k, KER_B), EV(k, KER_E)));
            stats->kernel_ms += ms;
            PIER_HIP(hipEventElapsedTime(&ms, EV(k, D2H_B), EV(k, D2H_E)));
            stats->d2h_ms += ms;
        }
        float wall = 0.f;
        PIER_HIP(hipEventElapsedTime(&wall, EV(0, H2D_B), EV(n_pieces - 1, D2H_E)));
        stats->wall_ms = wall;
        PIER_HIP(hipEventElapsedTime(&wall, EV(0, H2D_B), EV(n_pieces - 1, KER_E)));
        stats->compute_ms = wall;
    }
    return PIER_OK;
}

pier_status pier_offload_stream(pier_ctx* c, const pier_outer_hp* hp, size_t chunk_bytes,
                                void* workspace, size_t workspace_bytes, void* compute_stream,
                                void* h2d_stream, void* d2h_stream, pier_offload_stats* stats)
{
    OffloadSetup S;
    const pier_status st = offload_validate(c, hp, chunk_bytes, workspace, workspace_bytes, &S);
    if (st != PIER_OK) return st;
    return offload_enqueue(c, hp, S, workspace, compute_stream, h2d_stream, d2h_stream, stats);
}

float pier_mu_schedule(int64_t t, int64_t T)
{
    if (10 * t >= T && 100 * t < 15 * T) return 0.99f;
    if (100 * t >= 15 * T && 10 * t < 2 * T) return 0.95f;
    return 0.9f;
}

float pier_outer_lr_schedule(int64_t t, int64_t T)
{
    if (10 * t < T) return 0.0f;
    if (10 * t < 2 * T) return static_cast<float>(static_cast<double>(10 * t - T) / static_cast<double>(T));
    if (10 * t < 8 * T) return 1.1f;
    return 0.9f;
}

float pier_inner_lr_schedule(int64_t t, int64_t T, float lr_max, float lr_min, double warmup_frac)
{
    const double kPi = 3.14159265358979323846;
    const double W = warmup_frac * static_cast<double>(T);
    if (W > 0.0 && static_cast<double>(t) <= W)
        return static_cast<float>(static_cast<double>(lr_max) * static_cast<double>(t) / W);
    if (t >= T) return lr_min;
    const double ratio = (static_cast<double>(t) - W) / (static_cast<double>(T) - W);
    const double coeff = 0.5 * (std::cos(kPi * ratio) + 1.0);
    return static_cast<float>(static_cast<double>(lr_min) +
                              coeff * (static_cast<double>(lr_max) - static_cast<double>(lr_min)));
}

pier_status pier_train_step(pier_ctx* c, const pier_train_cfg* cfg, int64_t t, void* hip_stream)
{
    if (!c) return fail(PIER_ERR_INVALID_ARG, "ctx is NULL");
    if (!cfg) return fail(PIER_ERR_INVALID_ARG, "cfg is NULL");
    if (cfg->T < 1 || cfg->r < 1 || t < 1 || t > cfg->T)
        return fail(PIER_ERR_INVALID_ARG, "need T >= 1, r >= 1, 1 <= t <= T (T = %lld, r = %lld, t = %lld)",
                    static_cast<long long>(cfg->T), static_cast<long long>(cfg->r), static_cast<long long>(t));
    if (cfg->mode != PIER_MODE_PIER && cfg->mode != PIER_MODE_DILOCO)
        return fail(PIER_ERR_INVALID_ARG, "cfg->mode is neither PIER nor DILOCO");
    if (!(cfg->warmup_frac >= 0.0 && cfg->warmup_frac < 1.0) || !(cfg->clip_norm >= 0.0f))
        return fail(PIER_ERR_INVALID_ARG, "warmup_frac must lie in [0, 1) and clip_norm be >= 0");
    pier_status st = check_all_bound(c);
    if (st != PIER_OK) return st;
    const bool sync = (t % cfg->r) == 0;
    if (sync && !c->outer_bound) return fail(PIER_ERR_STATE, "anchor and momentum are not bound");

    pier_adamw_hp hp;
    hp.lr = pier_inner_lr_schedule(t, cfg->T, cfg->lr_max, cfg->lr_min, cfg->warmup_frac);
    hp.beta1 = cfg->beta1;
    hp.beta2 = cfg->beta2;
    hp.eps = cfg->eps;
    hp.weight_decay = cfg->weight_decay;
    hp.grad_scale = 1.0f;
    hp.step = t;
    const ClipMode clip = cfg->clip_norm > 0.0f ? kClipCtx : kNoClip;

    // Everything that can be refused is checked before the first launch: the inner step of every
    // replica and, on a synchronisation iteration, the whole outer step (bindings, working-copy
    // rule, offload piece size, workspace, chunking tables).
    for (int g = 0; g < c->n_replicas; ++g)
        if ((st = inner_adamw_validate(c, g, &hp, clip, cfg->clip_norm)) != PIER_OK) return st;
    pier_outer_hp ohp;
    OffloadSetup S;
    bool shadow = false;
    const bool offloaded = sync && c->outer_loc == PIER_LOC_HOST_PINNED;
    if (sync) {
        if (cfg->mode == PIER_MODE_DILOCO) {
            ohp.phase = PIER_PHASE_PIER;   // no lazy start; the DiLoCo paper's recommended scalars
            ohp.mu = 0.9f;
            ohp.outer_lr = 0.7f;
        } else if ((st = pier_outer_schedule(t, cfg->T, &ohp)) != PIER_OK) {
            return st;
        }
        st = offloaded ? offload_validate(c, &ohp, cfg->chunk_bytes, cfg->workspace, cfg->workspace_bytes, &S)
                       : outer_step_validate(c, &ohp, &shadow);
        if (st != PIER_OK) return st;
    }

    for (int g = 0; g < c->n_replicas; ++g)
        if ((st = inner_adamw_enqueue(c, g, &hp, clip, cfg->clip_norm, hip_stream)) != PIER_OK) return st;
    if (!sync) return PIER_OK;
    if (offloaded)
        return offload_enqueue(c, &ohp, S, cfg->workspace, hip_stream, cfg->h2d_stream, cfg->d2h_stream, nullptr);
    PIER_HIP(launch_outer(c->d_chunks, c->n_chunks, c->d_rows, c->n_replicas, nullptr, nullptr, 0, ohp.mu,
                          ohp.outer_lr, ohp.phase == PIER_PHASE_PIER, shadow, c->shape,
                          static_cast<hipStream_t>(hip_stream)));
    return PIER_OK;
}

pier_status pier_outer_schedule(int64_t t, int64_t T, pier_outer_hp* out)
{
    if (!out) return fail(PIER_ERR_INVALID_ARG, "out is NULL");
    if (T < 1 || t < 1 || t > T)
        return fail(PIER_ERR_INVALID_ARG, "need 1 <= t <= T (t = %lld, T = %lld)", static_cast<long long>(t),
                    static_cast<long long>(T));
    if (10 * t <= T) {
        out->phase = PIER_PHASE_WARMUP;
        out->mu = 0.9f;
        out->outer_lr = 0.0f;
    } else {
        out->phase = PIER_PHASE_PIER;
        out->mu = pier_mu_schedule(t, T);
        out->outer_lr = pier_outer_lr_schedule(t, T);
    }
    return PIER_OK;
}

}  // extern "C"
