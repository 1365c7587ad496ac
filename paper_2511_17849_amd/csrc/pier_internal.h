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

// Per-tensor pointers of one replica.  w: bfloat16 working copy of p (may be null).
struct RepPtrs {
    float* p;
    float* m;
    float* v;
    const void* g;
    unsigned short* w;
    void* reserved;
};

// Per-tensor row of the outer step's table: 4 + 2G eight-byte words, contiguous so that
// a workgroup fetches everything it needs about its tensor with one scalar load:
//   word 0: anchor pointer   word 1: momentum pointer
//   word 2: flat_start = number of elements in the tensors before this one (its
//           position in the flat host arrays of the offload path)
//   word 3: flags, bit 0 = every bound theta pointer of the tensor is 16-byte aligned,
//           bit 1 = every bound working-copy pointer is 8-byte aligned
//   words 4 .. 4+G-1: theta pointers of replicas 0 .. G-1
//   words 4+G .. 4+2G-1: bfloat16 working-copy pointers of the replicas (or null)
constexpr int kOuterRowHead = 4;
inline size_t outer_row_words(int G) { return static_cast<size_t>(kOuterRowHead + 2 * G); }

struct AdamwScalars {
    float lr, beta1, beta2, om1, om2, eps, wd, bc1, bc2, grad_scale;
};

struct LaunchShape {
    int unroll;       // 1, 2 or 4 vectors per lane per stream (workgroups of kBlock threads only)
    int max_grid;     // 0 = one chunk per team of kBlock lanes
    int nontemporal;  // 0 / 1
    int wg_threads;   // kBlock, or 64: a team is four one-wave workgroups; 0 = the kernel's best
    int lds_bytes;    // unused dynamic LDS per workgroup: caps the workgroups resident per CU; -1 = the kernel's best
};

constexpr int kBlock = 256;  // lanes that share one chunk: four 64-wide wavefronts

// Result of the gradient-norm pass of one replica (device memory).
struct ClipState {
    double sumsq;  // sum of squares of every gradient element
    double norm;   // its square root
    float coef;    // min(1, max_norm / (norm + 1e-6))
    float reserved;
};

constexpr int kDefaultNormPartials = 16384;  // workgroups (= partial sums) of the norm pass unless set otherwise

// clip: nullptr, or the replica's ClipState whose coef multiplies grad_scale.
// shadow: also write bfloat16(theta) through RepPtrs::w.
hipError_t launch_adamw(const Chunk* chunks, int n_chunks, const RepPtrs* tab, bool grad_bf16,
                        bool shadow, const AdamwScalars& s, const ClipState* clip,
                        const LaunchShape& shape, hipStream_t stream);

// Sum of squares of a replica's gradients: n_partials workgroups
// write one double each, then one workgroup folds them and the clip coefficient into *out.
hipError_t launch_grad_norm(const Chunk* chunks, int n_chunks, const RepPtrs* tab, bool grad_bf16,
                            double* partials, int n_partials, float max_norm, ClipState* out,
                            hipStream_t stream);

// rows: n_tensors rows of outer_row_words(G) words.  When flat_a != nullptr the anchor
// and momentum of element e of the flat index space are flat_a[e - flat_lo] and
// flat_M[e - flat_lo] (staging slot of an offload piece) and the rows supply only
// flat_start and the theta pointers; otherwise words 0 and 1 are used.
// shadow (Pier phase only): also write bfloat16(theta) to every replica's working copy.
hipError_t launch_outer(const Chunk* chunks, int n_chunks, const uint64_t* rows, int G,
                        float* flat_a, float* flat_M, int64_t flat_lo, float mu, float lr,
                        bool pier_phase, bool shadow, const LaunchShape& shape, hipStream_t stream);

// Two-stream in-place streaming pass used by the placement probe: reads n4 16-byte
// vectors from x and y, writes them back to where they came from.
hipError_t launch_probe(float* x, float* y, int64_t n4, hipStream_t stream);

}  // namespace pier
