// Internal declarations shared by the kernel file and the host-side API file of
// libpier.  Not part of the ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pier {

// One unit of work for a workgroup: `len` consecutive elements of tensor `tensor`
// starting at element `off`.  Chunks never cross a tensor boundary (nor, in the
// offload chunking, a piece boundary).
struct Chunk {
    int64_t off;
    int32_t tensor;
    int32_t len;
};
static_assert(sizeof(Chunk) == 16, "chunk entries are read as one 16-byte load");

// Per-tensor pointers of one replica.
struct RepPtrs {
    float* p;
    float* m;
    float* v;
    const void* g;
};

// Per-tensor outer state.  flat_start = number of elements in the tensors before
// this one (its position in the flat host arrays of the offload path).
struct OuterPtrs {
    float* a;
    float* M;
    int64_t flat_start;
    int64_t reserved;
};

struct AdamwScalars {
    float lr, beta1, beta2, om1, om2, eps, wd, bc1, bc2, grad_scale;
};

struct LaunchShape {
    int unroll;       // 1, 2 or 4
    int max_grid;     // 0 = one chunk per workgroup
    int nontemporal;  // 0 / 1
};

constexpr int kBlock = 256;  // four 64-wide wavefronts

hipError_t launch_adamw(const Chunk* chunks, int n_chunks, const RepPtrs* tab, bool grad_bf16,
                        const AdamwScalars& s, const LaunchShape& shape, hipStream_t stream);

// rep_tab holds G * n_tensors entries, replica-major.  When flat_a != nullptr the
// anchor and momentum of element e of the flat index space are flat_a[e - flat_lo]
// and flat_M[e - flat_lo] (staging slot of an offload piece) and otab supplies only
// flat_start; otherwise they are otab[tensor].a / .M.
hipError_t launch_outer(const Chunk* chunks, int n_chunks, const RepPtrs* rep_tab, int n_tensors,
                        int G, const OuterPtrs* otab, float* flat_a, float* flat_M,
                        int64_t flat_lo, float mu, float lr, bool pier_phase,
                        const LaunchShape& shape, hipStream_t stream);

}  // namespace pier
