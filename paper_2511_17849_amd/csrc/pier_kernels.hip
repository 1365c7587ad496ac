// HIP kernels of libpier for gfx950 (MI355X): the fused multi-tensor inner AdamW
// step and the fused outer step of Pier's two-level optimizer.
//
// Both kernels are elementwise streams bound by HBM bandwidth, so the design is:
//   * a team of 4 wavefronts per chunk of a tensor (chunk table in device memory, read
//     through the scalar unit because the index is wave-uniform), launched as one
//     workgroup or, by default, as four one-wave workgroups with a cap on the waves
//     resident per compute unit: both kernels stream faster with few waves in flight;
//   * 128-bit loads/stores, lane i of a wavefront touching vector i of a 1 KiB run,
//     so every wave-level access is one fully coalesced 1 KiB burst per stream;
//   * all loads of a tile (UNROLL vectors x every stream) are issued before the
//     first use, so each lane keeps UNROLL x streams 16-byte requests in flight;
//   * every buffer is read once and written once per launch; nothing is staged in
//     LDS because no element is shared between lanes (the sum over the G replicas
//     is a per-lane register reduction: replica g's element i lives at the same
//     index i of a different stream);
//   * no MFMA: there is no contraction anywhere on this path.
// Arithmetic is written in the order the update rules are stated, one fp32
// operation per operator, with FMA contraction switched off and correctly rounded
// division and square root, so results do not depend on how the compiler schedules
// the expression.
#include "pier_internal.h"

#include <cstddef>
#include <type_traits>

namespace pier {

typedef float vfloat4 __attribute__((ext_vector_type(4)));
typedef unsigned short vushort4 __attribute__((ext_vector_type(4)));

// Every pointer the kernels follow comes out of a table in memory, so the compiler
// cannot tell it addresses global memory and would fall back to flat instructions.
// All accesses therefore go through these helpers, which cast to the global address
// space (global_load / global_store) and apply the streaming hint.
#define PIER_GLOBAL __attribute__((address_space(1)))

template <bool NT, typename T>
__device__ __forceinline__ T ld(const T* p)
{
    const PIER_GLOBAL T* q = (const PIER_GLOBAL T*)p;
    if constexpr (NT) return __builtin_nontemporal_load(q);
    else return *q;
}

template <bool NT, typename T>
__device__ __forceinline__ void st(T* p, T x)
{
    PIER_GLOBAL T* q = (PIER_GLOBAL T*)p;
    if constexpr (NT) __builtin_nontemporal_store(x, q);
    else *q = x;
}

// Vector access at base + byte_off with a wave-uniform base and a 32-bit per-lane byte
// offset: this shape lets the compiler keep the base in SGPRs and one offset VGPR for all
// streams (global_load_dwordx4 v, v_off, s[base]) instead of a 64-bit VGPR address per stream.
template <bool NT, typename T>
__device__ __forceinline__ T ldo(const void* base, unsigned byte_off)
{
    return ld<NT>(reinterpret_cast<const T*>(static_cast<const char*>(base) + byte_off));
}

template <bool NT, typename T>
__device__ __forceinline__ void sto(void* base, unsigned byte_off, T x)
{
    st<NT>(reinterpret_cast<T*>(static_cast<char*>(base) + byte_off), x);
}

__device__ __forceinline__ float bf16_to_f32(unsigned short h)
{
    return __uint_as_float(static_cast<unsigned int>(h) << 16);
}

// fp32 -> bfloat16, round to nearest even; NaN becomes the quiet NaN 0x7FC0.  This is
// the working weight the model computes with (BF16 in models, FP32 in optimizers).
__device__ __forceinline__ unsigned short f32_to_bf16(float f)
{
    const unsigned int b = __float_as_uint(f);
    const unsigned int r = (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
    return static_cast<unsigned short>((b & 0x7FFFFFFFu) > 0x7F800000u ? 0x7FC0u : r);
}

__device__ __forceinline__ vushort4 f32_to_bf16(vfloat4 f)
{
    vushort4 r;
    r.x = f32_to_bf16(f.x);
    r.y = f32_to_bf16(f.y);
    r.z = f32_to_bf16(f.z);
    r.w = f32_to_bf16(f.w);
    return r;
}

// A chunk is always worked on by a team of kBlock lanes.  The team is one workgroup of
// kBlock threads, or kBlock / WG consecutive smaller workgroups (WG = 64: four one-wave
// workgroups), which the dispatcher deals to different XCDs and which retire one by one;
// the addresses each lane touches are the same either way.
template <int WG>
struct Team {
    static_assert(WG == 64 || WG == kBlock, "workgroups of one wave or of a whole team");
    static constexpr int kSplit = kBlock / WG;
    int lane;    // position of this thread among the kBlock lanes of its team
    int first;   // first chunk of the team
    int stride;  // teams in the grid
    __device__ __forceinline__ Team()
        : lane(static_cast<int>(blockIdx.x % kSplit) * WG + static_cast<int>(threadIdx.x)),
          first(static_cast<int>(blockIdx.x / kSplit)),
          stride(static_cast<int>(gridDim.x / kSplit))
    {
    }
};

// ------------------------------------------------------------------ inner AdamW
//
// AdamW with decoupled weight decay and bias correction (the inner optimizer of
// Algorithm 1 / Algorithm 2, hyper-parameters of Table I).
__device__ __forceinline__ void adamw_elem(float& p, float& m, float& v, float g,
                                           const AdamwScalars& s)
{
#pragma clang fp contract(off)
    g = g * s.grad_scale;
    const float mn = s.beta1 * m + s.om1 * g;
    const float vn = s.beta2 * v + (s.om2 * g) * g;
    const float mh = mn / s.bc1;
    const float vh = vn / s.bc2;
    const float u = mh / (sqrtf(vh) + s.eps) + s.wd * p;
    p = p - s.lr * u;
    m = mn;
    v = vn;
}

template <bool BF16>
struct GradVec;
template <>
struct GradVec<false> {
    typedef vfloat4 type;
    static __device__ __forceinline__ vfloat4 widen(vfloat4 x) { return x; }
};
template <>
struct GradVec<true> {
    typedef vushort4 type;
    static __device__ __forceinline__ vfloat4 widen(vushort4 x)
    {
        vfloat4 r;
        r.x = bf16_to_f32(x.x);
        r.y = bf16_to_f32(x.y);
        r.z = bf16_to_f32(x.z);
        r.w = bf16_to_f32(x.w);
        return r;
    }
};

__device__ __forceinline__ void adamw_vec(vfloat4& P, vfloat4& M, vfloat4& V, const vfloat4& G,
                                          const AdamwScalars& s)
{
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float p = P[k], m = M[k], v = V[k];
        adamw_elem(p, m, v, G[k], s);
        P[k] = p;
        M[k] = m;
        V[k] = v;
    }
}

template <bool BF16, bool SHADOW, typename GS>
__device__ __forceinline__ void adamw_scalar(float* p, float* m, float* v, const GS* g,
                                             unsigned short* w, const AdamwScalars& s)
{
    float pi = ld<false>(p), mi = ld<false>(m), vi = ld<false>(v), gi;
    if constexpr (BF16) gi = bf16_to_f32(ld<false>(g)); else gi = ld<false>(g);
    adamw_elem(pi, mi, vi, gi, s);
    st<false>(p, pi);
    st<false>(m, mi);
    st<false>(v, vi);
    if constexpr (SHADOW) st<false>(w, f32_to_bf16(pi));
}

template <int WG, int UNROLL, bool BF16, bool NT, bool SHADOW>
__global__ __launch_bounds__(WG) void adamw_kernel(const Chunk* __restrict__ chunks,
                                                   int n_chunks,
                                                   const RepPtrs* __restrict__ tab,
                                                   const ClipState* __restrict__ clip,
                                                   AdamwScalars s)
{
    // gradient clipping: the coefficient of the norm pass that ran before this launch
    if (clip) s.grad_scale = s.grad_scale * clip->coef;
    typedef typename GradVec<BF16>::type gvec;
    typedef typename std::conditional<BF16, unsigned short, float>::type gscalar;
    const Team<WG> team;
    const int tid = team.lane;
    constexpr int kTile = kBlock * UNROLL;  // vectors per tile

    for (int c = team.first; c < n_chunks; c += team.stride) {
        const Chunk ch = chunks[c];
        const RepPtrs t = tab[ch.tensor];
        float* __restrict__ p = t.p + ch.off;
        float* __restrict__ m = t.m + ch.off;
        float* __restrict__ v = t.v + ch.off;
        const gscalar* __restrict__ g = static_cast<const gscalar*>(t.g) + ch.off;
        unsigned short* __restrict__ w = SHADOW ? t.w + ch.off : nullptr;
        const int len = ch.len;

        const uintptr_t mis = (reinterpret_cast<uintptr_t>(p) | reinterpret_cast<uintptr_t>(m) |
                               reinterpret_cast<uintptr_t>(v)) & 15u;
        const uintptr_t gmis = (reinterpret_cast<uintptr_t>(g) & (sizeof(gvec) - 1)) |
                               (reinterpret_cast<uintptr_t>(w) & 7u);
        if ((mis | gmis) == 0) {
            constexpr unsigned kG = sizeof(gvec);
            const int n4 = len >> 2;
            int base = 0;
            for (; base + kTile <= n4; base += kTile) {
                vfloat4 P[UNROLL], M[UNROLL], V[UNROLL];
                gvec Gr[UNROLL];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    const unsigned i = static_cast<unsigned>(base + u * kBlock + tid);
                    P[u] = ldo<NT, vfloat4>(p, i * 16u);
                    M[u] = ldo<NT, vfloat4>(m, i * 16u);
                    V[u] = ldo<NT, vfloat4>(v, i * 16u);
                    Gr[u] = ldo<NT, gvec>(g, i * kG);
                }
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    const unsigned i = static_cast<unsigned>(base + u * kBlock + tid);
                    adamw_vec(P[u], M[u], V[u], GradVec<BF16>::widen(Gr[u]), s);
                    sto<NT>(p, i * 16u, P[u]);
                    sto<NT>(m, i * 16u, M[u]);
                    sto<NT>(v, i * 16u, V[u]);
                    if constexpr (SHADOW) sto<NT>(w, i * 8u, f32_to_bf16(P[u]));
                }
            }
            // ragged last tile of the chunk
            for (int j = base + tid; j < n4; j += kBlock) {
                const unsigned i = static_cast<unsigned>(j);
                vfloat4 P = ldo<NT, vfloat4>(p, i * 16u), M = ldo<NT, vfloat4>(m, i * 16u),
                        V = ldo<NT, vfloat4>(v, i * 16u);
                const gvec Gr = ldo<NT, gvec>(g, i * kG);
                adamw_vec(P, M, V, GradVec<BF16>::widen(Gr), s);
                sto<NT>(p, i * 16u, P);
                sto<NT>(m, i * 16u, M);
                sto<NT>(v, i * 16u, V);
                if constexpr (SHADOW) sto<NT>(w, i * 8u, f32_to_bf16(P));
            }
            // up to three elements past the last whole vector
            const int i = (n4 << 2) + tid;
            if (i < len) adamw_scalar<BF16, SHADOW>(p + i, m + i, v + i, g + i, w + i, s);
        } else {
            for (int i = tid; i < len; i += kBlock)
                adamw_scalar<BF16, SHADOW>(p + i, m + i, v + i, g + i, w + i, s);
        }
    }
}

static int grid_for(int n_chunks, const LaunchShape& shape)
{
    if (shape.max_grid > 0 && n_chunks > shape.max_grid) return shape.max_grid;
    return n_chunks;
}

// Fills in the fields of a launch shape left on "auto".  Measured on MI355X at GPT-2
// small .. 7B sizes: both kernels stream fastest with one-wave workgroups and only as
// many waves resident as their arithmetic needs to hide its own latency (more waves in
// flight spread the DRAM traffic over more open pages and read/write turnarounds):
// 12 waves per compute unit for AdamW (three divisions and a square root per element),
// 8 for the outer step, 20 for the lazy-start pass (three loads per lane, almost no
// arithmetic: 6.55 TB/s against 6.38 at 12 and 6.13 at 8).  The cap is an unused LDS
// reservation per workgroup.
static LaunchShape resolved(LaunchShape shape, int auto_lds)
{
    if (shape.wg_threads == 0) shape.wg_threads = (shape.unroll == 1 && shape.max_grid == 0) ? 64 : kBlock;
    if (shape.lds_bytes < 0) shape.lds_bytes = shape.wg_threads == 64 ? auto_lds : 0;
    return shape;
}
constexpr int kAdamwAutoLds = 13 * 1024;  // floor(160 KiB / 13 KiB) = 12 one-wave workgroups per CU
constexpr int kOuterAutoLds = 18 * 1024;  // 8 per CU
constexpr int kLazyAutoLds = 8 * 1024;    // 20 per CU: the lazy-start pass keeps only three loads per lane in flight

template <int WG, int U, bool BF16, bool SHADOW>
static void adamw_dispatch_nt(int grid, const Chunk* chunks, int n_chunks, const RepPtrs* tab,
                              const ClipState* clip, const AdamwScalars& s, const LaunchShape& shape,
                              hipStream_t stream)
{
    const dim3 g(static_cast<unsigned>(grid) * (kBlock / WG)), b(WG);
    const unsigned lds = static_cast<unsigned>(shape.lds_bytes);
    if (shape.nontemporal) hipLaunchKernelGGL((adamw_kernel<WG, U, BF16, true, SHADOW>), g, b, lds, stream,
                                              chunks, n_chunks, tab, clip, s);
    else hipLaunchKernelGGL((adamw_kernel<WG, U, BF16, false, SHADOW>), g, b, lds, stream,
                            chunks, n_chunks, tab, clip, s);
}

template <bool BF16, bool SHADOW>
static void adamw_dispatch_u(int grid, const Chunk* chunks, int n_chunks, const RepPtrs* tab,
                             const ClipState* clip, const AdamwScalars& s, const LaunchShape& shape,
                             hipStream_t stream)
{
    if (shape.wg_threads == 64) {   // one-wave workgroups: one vector per lane per stream only
        adamw_dispatch_nt<64, 1, BF16, SHADOW>(grid, chunks, n_chunks, tab, clip, s, shape, stream);
        return;
    }
    switch (shape.unroll) {
    case 1: adamw_dispatch_nt<kBlock, 1, BF16, SHADOW>(grid, chunks, n_chunks, tab, clip, s, shape, stream); break;
    case 2: adamw_dispatch_nt<kBlock, 2, BF16, SHADOW>(grid, chunks, n_chunks, tab, clip, s, shape, stream); break;
    default: adamw_dispatch_nt<kBlock, 4, BF16, SHADOW>(grid, chunks, n_chunks, tab, clip, s, shape, stream); break;
    }
}

hipError_t launch_adamw(const Chunk* chunks, int n_chunks, const RepPtrs* tab, bool grad_bf16,
                        bool shadow, const AdamwScalars& s, const ClipState* clip,
                        const LaunchShape& requested, hipStream_t stream)
{
    if (n_chunks <= 0) return hipSuccess;
    const LaunchShape shape = resolved(requested, kAdamwAutoLds);
    const int grid = grid_for(n_chunks, shape);
    if (grad_bf16) {
        if (shadow) adamw_dispatch_u<true, true>(grid, chunks, n_chunks, tab, clip, s, shape, stream);
        else adamw_dispatch_u<true, false>(grid, chunks, n_chunks, tab, clip, s, shape, stream);
    } else {
        if (shadow) adamw_dispatch_u<false, true>(grid, chunks, n_chunks, tab, clip, s, shape, stream);
        else adamw_dispatch_u<false, false>(grid, chunks, n_chunks, tab, clip, s, shape, stream);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------ gradient norm
//
// Global L2 norm of one replica's gradients for clipping (Table I, "clip grad 1"):
// squares are formed and accumulated in double (the product of two floats is exact in
// double), workgroup b folds chunks b, b + grid, b + 2 grid, ... in that order, lanes
// are folded by a fixed shuffle tree, and a second one-workgroup kernel folds the
// per-workgroup partial sums in a fixed order: no atomics, so the result is the same
// in every run of the same launch shape.
__device__ __forceinline__ double block_sum(double acc, double* lds)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_down(acc, off, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) lds[wave] = acc;
    __syncthreads();
    double total = 0.0;
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 0; w < kBlock / 64; ++w) total += lds[w];
    }
    return total;  // valid in thread 0
}

template <bool BF16>
__device__ __forceinline__ double sq4(typename GradVec<BF16>::type x)
{
    const vfloat4 f = GradVec<BF16>::widen(x);
    double a = static_cast<double>(f.x) * static_cast<double>(f.x);
    a += static_cast<double>(f.y) * static_cast<double>(f.y);
    a += static_cast<double>(f.z) * static_cast<double>(f.z);
    a += static_cast<double>(f.w) * static_cast<double>(f.w);
    return a;
}

template <bool BF16>
__global__ __launch_bounds__(kBlock) void sumsq_kernel(const Chunk* __restrict__ chunks, int n_chunks,
                                                       const RepPtrs* __restrict__ tab,
                                                       double* __restrict__ partials)
{
    typedef typename GradVec<BF16>::type gvec;
    typedef typename std::conditional<BF16, unsigned short, float>::type gscalar;
    __shared__ double lds[kBlock / 64];
    const int tid = threadIdx.x;
    double acc = 0.0;
    for (int c = blockIdx.x; c < n_chunks; c += gridDim.x) {
        const Chunk ch = chunks[c];
        const gscalar* __restrict__ g = static_cast<const gscalar*>(tab[ch.tensor].g) + ch.off;
        const int len = ch.len;
        if ((reinterpret_cast<uintptr_t>(g) & (sizeof(gvec) - 1)) == 0) {
            const int n4 = len >> 2;
            for (int j = tid; j < n4; j += kBlock)
                acc += sq4<BF16>(ldo<true, gvec>(g, static_cast<unsigned>(j) * static_cast<unsigned>(sizeof(gvec))));
            const int i = (n4 << 2) + tid;
            if (i < len) {
                float gi;
                if constexpr (BF16) gi = bf16_to_f32(ld<false>(g + i)); else gi = ld<false>(g + i);
                acc += static_cast<double>(gi) * static_cast<double>(gi);
            }
        } else {
            for (int i = tid; i < len; i += kBlock) {
                float gi;
                if constexpr (BF16) gi = bf16_to_f32(ld<false>(g + i)); else gi = ld<false>(g + i);
                acc += static_cast<double>(gi) * static_cast<double>(gi);
            }
        }
    }
    const double total = block_sum(acc, lds);
    if (tid == 0) partials[blockIdx.x] = total;
}

__global__ __launch_bounds__(kBlock) void clip_finalize_kernel(const double* __restrict__ partials,
                                                               int n_partials, float max_norm,
                                                               ClipState* __restrict__ out)
{
    __shared__ double lds[kBlock / 64];
    double acc = 0.0;
    for (int i = threadIdx.x; i < n_partials; i += kBlock) acc += partials[i];
    const double total = block_sum(acc, lds);
    if (threadIdx.x == 0) {
        const double norm = sqrt(total);
        const double coef = static_cast<double>(max_norm) / (norm + 1e-6);
        out->sumsq = total;
        out->norm = norm;
        out->coef = coef < 1.0 ? static_cast<float>(coef) : 1.0f;
        out->reserved = 0.0f;
    }
}

hipError_t launch_grad_norm(const Chunk* chunks, int n_chunks, const RepPtrs* tab, bool grad_bf16,
                            double* partials, int n_partials, float max_norm, ClipState* out,
                            hipStream_t stream)
{
    if (n_partials > n_chunks) n_partials = n_chunks;
    if (n_partials > 0) {
        if (grad_bf16) hipLaunchKernelGGL(sumsq_kernel<true>, dim3(n_partials), dim3(kBlock), 0, stream,
                                          chunks, n_chunks, tab, partials);
        else hipLaunchKernelGGL(sumsq_kernel<false>, dim3(n_partials), dim3(kBlock), 0, stream, chunks,
                                n_chunks, tab, partials);
    }
    hipLaunchKernelGGL(clip_finalize_kernel, dim3(1), dim3(kBlock), 0, stream, partials,
                       n_partials > 0 ? n_partials : 0, max_norm, out);
    return hipGetLastError();
}

// ------------------------------------------------------------------ outer step
//
// Algorithm 2, synchronisation branch, for one element held by G groups:
//   delta = (1/G) sum_g (theta_g - anchor);  M = mu M + delta;
//   theta = anchor + lr (mu M + delta), written to the anchor and to all groups.
// The sum over groups runs g = 0 .. G-1 in that order.
template <int G>
__device__ __forceinline__ void outer_elem(float (&th)[G], float& a, float& M, float mu, float lr,
                                           float invG)
{
#pragma clang fp contract(off)
    float s = 0.0f;
#pragma unroll
    for (int g = 0; g < G; ++g) s = s + (th[g] - a);
    const float d = s * invG;
    const float Mn = mu * M + d;
    M = Mn;
    const float x = a + lr * (mu * Mn + d);
    a = x;
#pragma unroll
    for (int g = 0; g < G; ++g) th[g] = x;
}

template <int G>
__device__ __forceinline__ void outer_vec(vfloat4 (&TH)[G], vfloat4& A, vfloat4& M, float mu,
                                          float lr, float invG)
{
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float th[G];
#pragma unroll
        for (int g = 0; g < G; ++g) th[g] = TH[g][k];
        float a = A[k], mm = M[k];
        outer_elem<G>(th, a, mm, mu, lr, invG);
        A[k] = a;
        M[k] = mm;
#pragma unroll
        for (int g = 0; g < G; ++g) TH[g][k] = th[g];
    }
}

template <int G, bool SHADOW>
__device__ __forceinline__ void outer_scalar(float* const (&th)[G], unsigned short* const (&wb)[G],
                                             float* a, float* M, int i, float mu, float lr, float invG)
{
    float t[G];
#pragma unroll
    for (int g = 0; g < G; ++g) t[g] = ld<false>(th[g] + i);
    float av = ld<false>(a + i), mv = ld<false>(M + i);
    outer_elem<G>(t, av, mv, mu, lr, invG);
    st<false>(a + i, av);
    st<false>(M + i, mv);
#pragma unroll
    for (int g = 0; g < G; ++g) st<false>(th[g] + i, t[g]);
    if constexpr (SHADOW) {
        const unsigned short h = f32_to_bf16(av);       // theta_g == new anchor for every g
#pragma unroll
        for (int g = 0; g < G; ++g) st<false>(wb[g] + i, h);
    }
}

struct OuterArgs {
    float* flat_a;
    float* flat_M;
    int64_t flat_lo;
    int n_chunks;
    int G;
    int shadow;
    float mu, lr, invG;
};

// One row of the outer table as the kernel for G replicas sees it.
template <int G>
struct OuterRow {
    float* a;
    float* M;
    int64_t flat_start;
    uint64_t flags;     // alignment summary for the kernel of arbitrary group counts
    float* th[G];
    unsigned short* wb[G];
};

// The tables are separate const __restrict__ parameters: only then may the compiler
// read them through the scalar unit (they are never written by a kernel).
template <int WG, int G, int UNROLL, bool FLAT, bool NT, bool SHADOW>
__global__ __launch_bounds__(WG) void outer_kernel(const Chunk* __restrict__ chunks,
                                                   const OuterRow<G>* __restrict__ rows,
                                                   OuterArgs A)
{
    const Team<WG> team;
    const int tid = team.lane;
    constexpr int kTile = kBlock * UNROLL;

    for (int c = team.first; c < A.n_chunks; c += team.stride) {
        const Chunk ch = chunks[c];
        const OuterRow<G> row = rows[ch.tensor];
        float* __restrict__ a;
        float* __restrict__ M;
        if constexpr (FLAT) {
            const int64_t e = row.flat_start + ch.off - A.flat_lo;
            a = A.flat_a + e;
            M = A.flat_M + e;
        } else {
            a = row.a + ch.off;
            M = row.M + ch.off;
        }
        float* th[G];
        unsigned short* wb[G];
        uintptr_t mis = reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(M);
        uintptr_t wmis = 0;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            th[g] = row.th[g] + ch.off;
            mis |= reinterpret_cast<uintptr_t>(th[g]);
            wb[g] = SHADOW ? row.wb[g] + ch.off : nullptr;
            wmis |= reinterpret_cast<uintptr_t>(wb[g]);
        }
        const int len = ch.len;

        if (((mis & 15u) | (wmis & 7u)) == 0) {
            const int n4 = len >> 2;
            int base = 0;
            for (; base + kTile <= n4; base += kTile) {
                vfloat4 TH[UNROLL][G], Av[UNROLL], Mv[UNROLL];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    const unsigned o = static_cast<unsigned>(base + u * kBlock + tid) * 16u;
                    Av[u] = ldo<NT, vfloat4>(a, o);
                    Mv[u] = ldo<NT, vfloat4>(M, o);
#pragma unroll
                    for (int g = 0; g < G; ++g) TH[u][g] = ldo<NT, vfloat4>(th[g], o);
                }
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    const unsigned o = static_cast<unsigned>(base + u * kBlock + tid) * 16u;
                    outer_vec<G>(TH[u], Av[u], Mv[u], A.mu, A.lr, A.invG);
                    sto<NT>(a, o, Av[u]);
                    sto<NT>(M, o, Mv[u]);
#pragma unroll
                    for (int g = 0; g < G; ++g) sto<NT>(th[g], o, TH[u][g]);
                    if constexpr (SHADOW) {
                        const vushort4 h = f32_to_bf16(Av[u]);
#pragma unroll
                        for (int g = 0; g < G; ++g) sto<NT>(wb[g], o >> 1, h);
                    }
                }
            }
            for (int j = base + tid; j < n4; j += kBlock) {
                const unsigned o = static_cast<unsigned>(j) * 16u;
                vfloat4 TH[G], Av = ldo<NT, vfloat4>(a, o), Mv = ldo<NT, vfloat4>(M, o);
#pragma unroll
                for (int g = 0; g < G; ++g) TH[g] = ldo<NT, vfloat4>(th[g], o);
                outer_vec<G>(TH, Av, Mv, A.mu, A.lr, A.invG);
                sto<NT>(a, o, Av);
                sto<NT>(M, o, Mv);
#pragma unroll
                for (int g = 0; g < G; ++g) sto<NT>(th[g], o, TH[g]);
                if constexpr (SHADOW) {
                    const vushort4 h = f32_to_bf16(Av);
#pragma unroll
                    for (int g = 0; g < G; ++g) sto<NT>(wb[g], o >> 1, h);
                }
            }
            const int i = (n4 << 2) + tid;
            if (i < len) outer_scalar<G, SHADOW>(th, wb, a, M, i, A.mu, A.lr, A.invG);
        } else {
            for (int i = tid; i < len; i += kBlock)
                outer_scalar<G, SHADOW>(th, wb, a, M, i, A.mu, A.lr, A.invG);
        }
    }
}

// Any number of groups: the replicas are walked in a run-time loop (same order, same
// arithmetic).  Where every stream of the chunk is 16-byte aligned (the host records that per
// tensor in word 3 of the row: bit 0 for the theta pointers, bit 1 for the working copies),
// lanes move 128-bit vectors and keep up to eight replica loads in flight; otherwise one
// element per lane.  Covers the group counts without a specialised kernel.
__device__ __forceinline__ void outer_anyG_scalar(const uint64_t* __restrict__ row, const OuterArgs& A,
                                                  float* a, float* M, int64_t off, int i)
{
#pragma clang fp contract(off)
    const float av = ld<false>(a + i);
    float s = 0.0f;
    for (int g = 0; g < A.G; ++g) {
        const float t = ld<false>(reinterpret_cast<const float*>(row[kOuterRowHead + g]) + off + i);
        s = s + (t - av);
    }
    const float d = s * A.invG;
    const float Mn = A.mu * ld<false>(M + i) + d;
    st<false>(M + i, Mn);
    const float x = av + A.lr * (A.mu * Mn + d);
    st<false>(a + i, x);
    for (int g = 0; g < A.G; ++g)
        st<false>(reinterpret_cast<float*>(row[kOuterRowHead + g]) + off + i, x);
    if (A.shadow) {
        const unsigned short h = f32_to_bf16(x);
        for (int g = 0; g < A.G; ++g)
            st<false>(reinterpret_cast<unsigned short*>(row[kOuterRowHead + A.G + g]) + off + i, h);
    }
}

template <int WG, bool FLAT, bool NT>
__global__ __launch_bounds__(WG) void outer_kernel_anyG(const Chunk* __restrict__ chunks,
                                                        const uint64_t* __restrict__ rows,
                                                        OuterArgs A)
{
#pragma clang fp contract(off)
    constexpr int kBatch = 8;   // replica loads in flight per lane
    const Team<WG> team;
    const int tid = team.lane;
    for (int c = team.first; c < A.n_chunks; c += team.stride) {
        const Chunk ch = chunks[c];
        const uint64_t* __restrict__ row = rows + static_cast<int64_t>(ch.tensor) * (kOuterRowHead + 2 * A.G);
        float* __restrict__ a;
        float* __restrict__ M;
        if constexpr (FLAT) {
            const int64_t e = static_cast<int64_t>(row[2]) + ch.off - A.flat_lo;
            a = A.flat_a + e;
            M = A.flat_M + e;
        } else {
            a = reinterpret_cast<float*>(row[0]) + ch.off;
            M = reinterpret_cast<float*>(row[1]) + ch.off;
        }
        const uint64_t flags = row[3];
        const bool vec = (flags & 1u) && (ch.off & 3) == 0 &&
                         ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(M)) & 15u) == 0 &&
                         (!A.shadow || (flags & 2u));
        if (vec) {
            const int n4 = ch.len >> 2;
            for (int j = tid; j < n4; j += kBlock) {
                const unsigned o = static_cast<unsigned>(j) * 16u;
                vfloat4 Av = ldo<NT, vfloat4>(a, o), Mv = ldo<NT, vfloat4>(M, o);
                vfloat4 s = {0.0f, 0.0f, 0.0f, 0.0f};
                for (int g0 = 0; g0 < A.G; g0 += kBatch) {
                    vfloat4 T[kBatch];
#pragma unroll
                    for (int k = 0; k < kBatch; ++k)
                        if (g0 + k < A.G)
                            T[k] = ldo<NT, vfloat4>(reinterpret_cast<const float*>(row[kOuterRowHead + g0 + k]) + ch.off, o);
#pragma unroll
                    for (int k = 0; k < kBatch; ++k)
                        if (g0 + k < A.G) s = s + (T[k] - Av);
                }
                const vfloat4 d = s * A.invG;
                const vfloat4 Mn = A.mu * Mv + d;
                sto<NT>(M, o, Mn);
                const vfloat4 x = Av + A.lr * (A.mu * Mn + d);
                sto<NT>(a, o, x);
                for (int g = 0; g < A.G; ++g)
                    sto<NT>(reinterpret_cast<float*>(row[kOuterRowHead + g]) + ch.off, o, x);
                if (A.shadow) {
                    const vushort4 h = f32_to_bf16(x);
                    for (int g = 0; g < A.G; ++g)
                        sto<NT>(reinterpret_cast<unsigned short*>(row[kOuterRowHead + A.G + g]) + ch.off, o >> 1, h);
                }
            }
            const int i = (n4 << 2) + tid;      // up to three elements past the last whole vector
            if (i < ch.len) outer_anyG_scalar(row, A, a, M, ch.off, i);
        } else {
            for (int i = tid; i < ch.len; i += kBlock) outer_anyG_scalar(row, A, a, M, ch.off, i);
        }
    }
}

// ------------------------------------------------------------------ lazy-start synchronisation
//
// Algorithm 1, the t mod r = 0 branch, for one element.  The algorithm is stated for one
// model (groups are formed only after the warmup), so the model is read from replica 0
// and nothing is averaged:
//   delta = theta - anchor;  M = mu M + delta;  anchor = theta.
// The model, its other replicas and their AdamW state are not touched.  Three streams
// read, two written: 20 bytes per parameter whatever the group count.
__device__ __forceinline__ void lazy_start_scalar(const float* th, float* a, float* M, int i, float mu)
{
#pragma clang fp contract(off)
    const float t = ld<false>(th + i);
    const float d = t - ld<false>(a + i);
    st<false>(M + i, mu * ld<false>(M + i) + d);
    st<false>(a + i, t);
}

template <int WG, bool FLAT, bool NT>
__global__ __launch_bounds__(WG) void lazy_start_kernel(const Chunk* __restrict__ chunks,
                                                        const uint64_t* __restrict__ rows,
                                                        OuterArgs A)
{
#pragma clang fp contract(off)
    const Team<WG> team;
    const int tid = team.lane;
    for (int c = team.first; c < A.n_chunks; c += team.stride) {
        const Chunk ch = chunks[c];
        const uint64_t* __restrict__ row = rows + static_cast<int64_t>(ch.tensor) * (kOuterRowHead + 2 * A.G);
        float* __restrict__ a;
        float* __restrict__ M;
        if constexpr (FLAT) {
            const int64_t e = static_cast<int64_t>(row[2]) + ch.off - A.flat_lo;
            a = A.flat_a + e;
            M = A.flat_M + e;
        } else {
            a = reinterpret_cast<float*>(row[0]) + ch.off;
            M = reinterpret_cast<float*>(row[1]) + ch.off;
        }
        const float* __restrict__ th = reinterpret_cast<const float*>(row[kOuterRowHead]) + ch.off;
        const uintptr_t mis = (reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(M) |
                               reinterpret_cast<uintptr_t>(th)) & 15u;
        if (mis == 0) {
            const int n4 = ch.len >> 2;
            for (int j = tid; j < n4; j += kBlock) {
                const unsigned o = static_cast<unsigned>(j) * 16u;
                const vfloat4 T = ldo<NT, vfloat4>(th, o), Av = ldo<NT, vfloat4>(a, o), Mv = ldo<NT, vfloat4>(M, o);
                const vfloat4 d = T - Av;
                sto<NT>(M, o, A.mu * Mv + d);
                sto<NT>(a, o, T);
            }
            const int i = (n4 << 2) + tid;      // up to three elements past the last whole vector
            if (i < ch.len) lazy_start_scalar(th, a, M, i, A.mu);
        } else {
            for (int i = tid; i < ch.len; i += kBlock) lazy_start_scalar(th, a, M, i, A.mu);
        }
    }
}

struct OuterTables {
    const Chunk* chunks;
    const uint64_t* rows;
};

// The uint64 table rows are handed to the register-array kernel as OuterRow<G>: same words,
// same order (the static_asserts below pin the layout the host writes).
template <int G>
static const OuterRow<G>* typed_rows(const uint64_t* rows)
{
    static_assert(std::is_standard_layout<OuterRow<G>>::value, "row must be plain data");
    static_assert(offsetof(OuterRow<G>, a) == 0 && offsetof(OuterRow<G>, M) == 8 &&
                  offsetof(OuterRow<G>, flat_start) == 16 && offsetof(OuterRow<G>, flags) == 24 &&
                  offsetof(OuterRow<G>, th) == 8 * kOuterRowHead &&
                  offsetof(OuterRow<G>, wb) == 8 * (kOuterRowHead + G) &&
                  sizeof(OuterRow<G>) == 8 * (kOuterRowHead + 2 * G) && sizeof(void*) == 8,
                  "OuterRow<G> must match the word layout of the outer table");
    return reinterpret_cast<const OuterRow<G>*>(rows);
}

template <int WG, int G, int U, bool FLAT, bool SHADOW>
static void outer_launch(int grid, const OuterTables& T, const OuterArgs& A, const LaunchShape& shape, hipStream_t stream)
{
    const OuterRow<G>* ROWS = typed_rows<G>(T.rows);
    const dim3 g(static_cast<unsigned>(grid) * (kBlock / WG)), b(WG);
    const unsigned lds = static_cast<unsigned>(shape.lds_bytes);
    if (shape.nontemporal) hipLaunchKernelGGL((outer_kernel<WG, G, U, FLAT, true, SHADOW>), g, b, lds, stream, T.chunks, ROWS, A);
    else hipLaunchKernelGGL((outer_kernel<WG, G, U, FLAT, false, SHADOW>), g, b, lds, stream, T.chunks, ROWS, A);
}

template <int WG, int G, int U, bool FLAT>
static void outer_dispatch_nt(int grid, const OuterTables& T, const OuterArgs& A, const LaunchShape& shape, hipStream_t stream)
{
    if (A.shadow) outer_launch<WG, G, U, FLAT, true>(grid, T, A, shape, stream);
    else outer_launch<WG, G, U, FLAT, false>(grid, T, A, shape, stream);
}

template <int G, bool FLAT>
static void outer_dispatch_u(int grid, const OuterTables& T, const OuterArgs& A, const LaunchShape& shape, hipStream_t stream)
{
    if (shape.wg_threads == 64) {   // one-wave workgroups: one vector per lane per stream only
        outer_dispatch_nt<64, G, 1, FLAT>(grid, T, A, shape, stream);
        return;
    }
    // lanes keep (G + 2) * unroll 16-byte loads in flight; cap the product
    int u = shape.unroll;
    while (u > 1 && (G + 2) * u > 20) u >>= 1;
    switch (u) {
    case 1: outer_dispatch_nt<kBlock, G, 1, FLAT>(grid, T, A, shape, stream); break;
    case 2: outer_dispatch_nt<kBlock, G, 2, FLAT>(grid, T, A, shape, stream); break;
    default:
        if constexpr ((G + 2) * 4 <= 20) outer_dispatch_nt<kBlock, G, 4, FLAT>(grid, T, A, shape, stream);
        else outer_dispatch_nt<kBlock, G, 2, FLAT>(grid, T, A, shape, stream);
        break;
    }
}

// One kernel template launched as one-wave or four-wave workgroups, streaming or cached.
#define PIER_LAUNCH_TEAM(KERNEL, FLAT_)                                                                    \
    do {                                                                                                   \
        const unsigned lds = static_cast<unsigned>(shape.lds_bytes);                                       \
        if (shape.wg_threads == 64) {                                                                      \
            const dim3 g(static_cast<unsigned>(grid) * (kBlock / 64)), b(64);                              \
            if (shape.nontemporal) hipLaunchKernelGGL((KERNEL<64, FLAT_, true>), g, b, lds, stream, T.chunks, T.rows, A);  \
            else hipLaunchKernelGGL((KERNEL<64, FLAT_, false>), g, b, lds, stream, T.chunks, T.rows, A);   \
        } else {                                                                                           \
            const dim3 g(static_cast<unsigned>(grid)), b(kBlock);                                          \
            if (shape.nontemporal) hipLaunchKernelGGL((KERNEL<kBlock, FLAT_, true>), g, b, lds, stream, T.chunks, T.rows, A); \
            else hipLaunchKernelGGL((KERNEL<kBlock, FLAT_, false>), g, b, lds, stream, T.chunks, T.rows, A); \
        }                                                                                                  \
    } while (0)

template <bool FLAT>
static void outer_dispatch_g(int grid, const OuterTables& T, const OuterArgs& A, const LaunchShape& shape, hipStream_t stream)
{
    // The register-array kernels are 1-10 % faster than the loop kernel at their group counts.
    switch (A.G) {
    case 1: outer_dispatch_u<1, FLAT>(grid, T, A, shape, stream); break;
    case 2: outer_dispatch_u<2, FLAT>(grid, T, A, shape, stream); break;
    case 4: outer_dispatch_u<4, FLAT>(grid, T, A, shape, stream); break;
    case 8: outer_dispatch_u<8, FLAT>(grid, T, A, shape, stream); break;
    default: PIER_LAUNCH_TEAM(outer_kernel_anyG, FLAT); break;
    }
}

hipError_t launch_outer(const Chunk* chunks, int n_chunks, const uint64_t* rows, int G,
                        float* flat_a, float* flat_M, int64_t flat_lo, float mu, float lr,
                        bool pier_phase, bool shadow, const LaunchShape& requested, hipStream_t stream)
{
    if (n_chunks <= 0) return hipSuccess;
    const LaunchShape shape = resolved(requested, pier_phase ? kOuterAutoLds : kLazyAutoLds);
    const OuterTables T{chunks, rows};
    OuterArgs A;
    A.flat_a = flat_a;
    A.flat_M = flat_M;
    A.flat_lo = flat_lo;
    A.n_chunks = n_chunks;
    A.G = G;
    A.shadow = (shadow && pier_phase) ? 1 : 0;
    A.mu = mu;
    A.lr = lr;
    A.invG = 1.0f / static_cast<float>(G);
    const int grid = grid_for(n_chunks, shape);
    const bool flat = flat_a != nullptr;
    if (pier_phase) {
        if (flat) outer_dispatch_g<true>(grid, T, A, shape, stream);
        else outer_dispatch_g<false>(grid, T, A, shape, stream);
    } else {
        if (flat) PIER_LAUNCH_TEAM(lazy_start_kernel, true);
        else PIER_LAUNCH_TEAM(lazy_start_kernel, false);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------ placement probe
//
// The access pattern of the two optimizer kernels reduced to its memory behaviour: every
// lane reads one vector from each of two buffers and writes both back in place (the sum
// keeps the loads alive; the buffers are scratch while a probe runs).
__global__ __launch_bounds__(kBlock) void probe_kernel(float* __restrict__ x, float* __restrict__ y,
                                                       int64_t n4)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= n4) return;
    vfloat4* x4 = reinterpret_cast<vfloat4*>(x);
    vfloat4* y4 = reinterpret_cast<vfloat4*>(y);
    const vfloat4 a = ld<true>(x4 + i), b = ld<true>(y4 + i);
    const vfloat4 s = a + b;
    st<true>(x4 + i, s);
    st<true>(y4 + i, s);
}

hipError_t launch_probe(float* x, float* y, int64_t n4, hipStream_t stream)
{
    if (n4 <= 0) return hipSuccess;
    const int64_t grid = (n4 + kBlock - 1) / kBlock;
    hipLaunchKernelGGL(probe_kernel, dim3(static_cast<unsigned>(grid)), dim3(kBlock), 0, stream, x, y, n4);
    return hipGetLastError();
}

}  // namespace pier
