// Placement of model-sized buffers in MI355X's HBM: the classifier of probe rates (pure host
// arithmetic), the probe that measures those rates on the GPU, and the placement plan.
// None of this is an operation of the paper; it is what lets the two kernels stream at
// their best rate whatever addresses the driver hands out.
#include "pier_host.h"
#include "pier_internal.h"

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <functional>
#include <vector>

using namespace pier;

namespace {

// ------------------------------------------------------------------ classification
//
// What the probe sees on MI355X: two granules streamed in place together run at one of two
// levels.  Granules of DIFFERENT address classes reach the top level, a band a few per cent
// wide under the best rate seen anywhere; granules of ONE class run below it, at a rate that
// swings with their distance (and neighbouring distances swing in opposite directions, so
// against two adjacent reference granules the slower pairing of a same-class granule is
// always clearly under the band).  Every threshold is a fraction of the best rate measured
// in the same run, so clock, memory speed and the kernel's efficiency cancel.
constexpr double kBand = 0.033;      // width of the top level: cross-class pairings lie within 3.3 % of the best rate seen
constexpr double kGap = 0.02;        // the two levels of the sweep must be at least 2 % of the best rate apart
constexpr double kBandShare = 0.15;  // ... and the top level must hold at least this share of the sweep (and two samples)
constexpr int kMaxClasses = 8;

// What the calling thread's most recent classification saw (pier_hbm_probe_summary).
struct ProbeSummary {
    double best = 0.0;        // fastest pairing
    double threshold = 0.0;   // level a pairing must reach to count as cross-class
    int n_classes = 0;
    int n_pairs = 0;          // pairings asked for
};
thread_local ProbeSummary g_summary;

// rate(a, b): streaming rate of granules a and b together (any unit, > 0), measured or
// looked up; n granules.  Returns false when rate() reported a failure (a value <= 0).
bool classify_granules(int n, const std::function<double(int, int)>& rate, int32_t* class_out)
{
    g_summary = ProbeSummary();
    bool ok = true;
    auto r = [&](int a, int b) {
        const double x = rate(a, b);
        if (!(x > 0.0)) ok = false;
        ++g_summary.n_pairs;
        if (x > g_summary.best) g_summary.best = x;
        return x;
    };
    // First sweep: granules 0 and 1 (adjacent, so of one class unless a class ends between them)
    // against granules across the arena.  Per sampled granule t: the slower and the faster of its
    // two pairings.  A granule of another class is fast against BOTH references; a granule of the
    // references' class is slow against at least one of them.
    struct Sample { double slower, faster; };
    std::vector<Sample> sweep;
    double fast = 0.0;
    const int stride = std::max(1, n / 24);
    for (int t = 2; t < n && ok; t += stride) {
        const double r0 = r(0, t), r1 = r(1, t);
        fast = std::max(fast, std::max(r0, r1));
        sweep.push_back({std::min(r0, r1), std::max(r0, r1)});
    }
    if (!ok) return false;
    // Sort by the slower pairing and look for the two levels: the widest gap under a top group of
    // at least `need` samples that starts inside the top band and is no wider than one and a half
    // bands.  Several classes iff that gap is wide enough - or every sample is in the band (the
    // references are alone in their class).
    bool one_class = true;
    double thr = (1.0 - kBand) * fast;
    if (!sweep.empty()) {
        std::sort(sweep.begin(), sweep.end(), [](const Sample& x, const Sample& y) { return x.slower > y.slower; });
        const size_t m = sweep.size();
        const size_t need = std::max<size_t>(2, static_cast<size_t>(kBandShare * static_cast<double>(m) + 0.999));
        const double floor_ = (1.0 - kBand) * fast;
        if (sweep[0].slower >= floor_ && sweep[0].slower - sweep[m - 1].slower <= 1.5 * kBand * fast) {
            one_class = false;                       // every sample at the top level
        } else {
            size_t split = 0;                        // top group = sweep[0 .. split)
            double gap = 0.0;
            for (size_t k = need; k < m; ++k) {
                // the top group must be one level: no wider than one and a half bands
                if (sweep[0].slower - sweep[k - 1].slower > 1.5 * kBand * fast) break;
                const double g = sweep[k - 1].slower - sweep[k].slower;
                if (g > gap) { gap = g; split = k; }
            }
            if (split > 0 && gap >= kGap * fast && sweep[0].slower >= floor_) {
                one_class = false;
                // the level a single pairing must reach to count as cross-class: half way between the
                // fastest pairing of any same-class sample and the slowest cross-class one
                double same_hi = 0.0;
                for (size_t k = split; k < m; ++k) same_hi = std::max(same_hi, sweep[k].faster);
                const double cross_lo = sweep[split - 1].slower;
                thr = same_hi < cross_lo ? 0.5 * (same_hi + cross_lo) : cross_lo - 0.25 * gap;
            }
        }
    }
    std::vector<std::vector<int>> classes;
    for (int t = 0; t < n && ok; ++t) {
        int pick = -1;
        double lowest = 1e300;
        if (one_class) {
            pick = classes.empty() ? -1 : 0;
        } else {
            for (size_t c = 0; c < classes.size() && ok; ++c) {
                // against the first and the latest member of the class; the slower pairing
                // decides (a few same-class distances stream almost as fast as cross-class pairs)
                const std::vector<int>& m = classes[c];
                double x = r(m.front(), t);
                if (m.back() != m.front() && x >= thr) x = std::min(x, r(m.back(), t));
                if (x < lowest) { lowest = x; pick = static_cast<int>(c); }
            }
        }
        if (pick >= 0 && (one_class || lowest < thr || classes.size() >= static_cast<size_t>(kMaxClasses)))
            classes[pick].push_back(t);
        else classes.push_back(std::vector<int>(1, t));
    }
    if (!ok) return false;
    for (size_t c = 0; c < classes.size(); ++c)
        for (int t : classes[c]) class_out[t] = static_cast<int32_t>(c);
    g_summary.threshold = one_class ? 0.0 : thr;
    g_summary.n_classes = static_cast<int>(classes.size());
    return true;
}

}  // namespace

extern "C" {

pier_status pier_hbm_classify(const double* rates, int n_granules, int32_t* class_out)
{
    if (!rates || !class_out) return fail(PIER_ERR_INVALID_ARG, "rates or class_out is NULL");
    if (n_granules < 2 || n_granules > 4096)
        return fail(PIER_ERR_INVALID_ARG, "n_granules = %d, need 2..4096", n_granules);
    const size_t n = static_cast<size_t>(n_granules);
    const bool ok = classify_granules(n_granules, [&](int a, int b) { return rates[a * n + b]; }, class_out);
    if (!ok) return fail(PIER_ERR_INVALID_ARG, "the rate table has an entry that is not a positive number");
    return PIER_OK;
}

pier_status pier_hbm_probe_summary(double* best_rate, double* threshold, int32_t* n_classes, int32_t* n_pairs)
{
    if (g_summary.n_pairs == 0 && g_summary.n_classes == 0)
        return fail(PIER_ERR_STATE, "this thread has not run pier_hbm_probe or pier_hbm_classify");
    if (best_rate) *best_rate = g_summary.best;
    if (threshold) *threshold = g_summary.threshold;
    if (n_classes) *n_classes = g_summary.n_classes;
    if (n_pairs) *n_pairs = g_summary.n_pairs;
    return PIER_OK;
}

pier_status pier_hbm_probe(void* arena, size_t bytes, size_t granule_bytes, int32_t* class_out,
                           int n_granules, void* hip_stream)
{
    if (!arena || !class_out) return fail(PIER_ERR_INVALID_ARG, "arena or class_out is NULL");
    const size_t kMiB = 1u << 20;
    if (granule_bytes < 512 * kMiB || granule_bytes % (2 * kMiB))
        return fail(PIER_ERR_INVALID_ARG, "granule_bytes must be a multiple of 2 MiB, at least 512 MiB");
    if (reinterpret_cast<uintptr_t>(arena) % 16) return fail(PIER_ERR_ALIGNMENT, "arena is not aligned to 16 bytes");
    if (n_granules < 2 || n_granules > 4096 || static_cast<size_t>(n_granules) > bytes / granule_bytes)
        return fail(PIER_ERR_INVALID_ARG, "n_granules = %d does not fit %zu bytes of %zu-byte granules (need 2..4096)",
                    n_granules, bytes, granule_bytes);
    int dev = -1;
    PIER_HIP(hipGetDevice(&dev));
    pier_status st = check_device_range(arena, static_cast<int64_t>(granule_bytes) * n_granules, 1, dev, "arena", 0);
    if (st != PIER_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    PIER_HIP(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return fail(PIER_ERR_HIP, "hipEventCreate failed");
    }
    // probe up to 2 GiB of each granule: far more than the 256 MB memory-side cache, and
    // long enough (> 1 ms per pass) that ramp-up and tail do not blur the two rate levels
    const size_t probe_bytes = std::min<size_t>(granule_bytes, 2048 * kMiB);
    const int64_t n4 = static_cast<int64_t>(probe_bytes / 16);
    char* base = static_cast<char*>(arena);
    auto granule = [&](int g) { return reinterpret_cast<float*>(base + static_cast<size_t>(g) * granule_bytes); };
    hipError_t err = hipSuccess;
    const bool verbose = std::getenv("PIER_PROBE_VERBOSE") != nullptr;
    // streaming rate (TB/s) of one in-place pass over granules a and b, faster of two; 0 on failure
    auto measure = [&](int a, int b) -> double {
        double bestr = 0.0;
        if (err == hipSuccess) err = launch_probe(granule(a), granule(b), n4, s);   // warm
        for (int r = 0; r < 2 && err == hipSuccess; ++r) {
            err = hipEventRecord(e0, s);
            if (err == hipSuccess) err = launch_probe(granule(a), granule(b), n4, s);
            if (err == hipSuccess) err = hipEventRecord(e1, s);
            if (err == hipSuccess) err = hipEventSynchronize(e1);
            float ms = 0.f;
            if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
            if (err == hipSuccess && ms > 0.f) bestr = std::max(bestr, 4.0 * probe_bytes / (ms * 1e9));
        }
        if (verbose) fprintf(stderr, "[pier probe] %d x %d: %.3f TB/s\n", a, b, bestr);
        return err == hipSuccess ? bestr : 0.0;
    };
    const bool ok = classify_granules(n_granules, measure, class_out);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (err != hipSuccess) return fail(PIER_ERR_HIP, "placement probe: %s", hipGetErrorString(err));
    if (!ok) return fail(PIER_ERR_HIP, "placement probe: a timed pass reported no duration");
    return PIER_OK;
}

pier_status pier_placement_plan(int n_classes, const int64_t* room_in, int n_replicas, int shared_grad,
                                int outer_on_device, pier_replica_placement* replicas,
                                int32_t* anchor_class, int32_t* momentum_class)
{
    if (n_classes < 1 || n_classes > 64) return fail(PIER_ERR_INVALID_ARG, "n_classes = %d, need 1..64", n_classes);
    if (!room_in || !replicas || !anchor_class || !momentum_class)
        return fail(PIER_ERR_INVALID_ARG, "a pointer is NULL");
    if (n_replicas < 1 || n_replicas > PIER_MAX_REPLICAS)
        return fail(PIER_ERR_INVALID_ARG, "n_replicas = %d, need 1..%d", n_replicas, PIER_MAX_REPLICAS);
    std::vector<int64_t> room(room_in, room_in + n_classes);
    for (int c = 0; c < n_classes; ++c)
        if (room[c] < 0) return fail(PIER_ERR_INVALID_ARG, "room[%d] is negative", c);
    const int two = std::min(2, n_classes);

    // takes `count` buffers from the first class of prefs[0..n_prefs) that holds them all, else
    // from the class with most room; -1 if no class holds them
    auto take = [&](const int* prefs, int n_prefs, int count) -> int {
        for (int i = 0; i < n_prefs; ++i)
            if (room[prefs[i]] >= count) {
                room[prefs[i]] -= count;
                return prefs[i];
            }
        int best = 0;
        for (int c = 1; c < n_classes; ++c)
            if (room[c] > room[best]) best = c;
        if (room[best] < count) return -1;
        room[best] -= count;
        return best;
    };
    auto full = [&]() { return fail(PIER_ERR_OOM, "the model's buffers do not fit the room given"); };

    std::vector<int> outer_load(n_classes, 0);
    for (int g = 0; g < n_replicas; ++g) {
        const int want[2] = {g % two, (g + 1) % two};
        int c = take(want, two, 2);                 // theta_g and m_g together
        if (c >= 0) {
            replicas[g].theta = replicas[g].m = c;
        } else {
            if ((replicas[g].theta = take(want, two, 1)) < 0) return full();
            if ((replicas[g].m = take(want, two, 1)) < 0) return full();
        }
        ++outer_load[replicas[g].theta];
    }
    *anchor_class = *momentum_class = -1;
    if (outer_on_device) {
        for (int32_t* out : {anchor_class, momentum_class}) {
            int lo = 0;
            for (int c = 1; c < two; ++c)
                if (outer_load[c] < outer_load[lo]) lo = c;
            const int want[2] = {lo, (lo + 1) % two};
            if ((*out = take(want, two, 1)) < 0) return full();
            ++outer_load[*out];
        }
    }
    int shared = -1;
    for (int g = 0; g < n_replicas; ++g) {
        // away from theta_g's class: class 2 first, then the other one of classes 0 and 1
        const int th = replicas[g].theta;
        int want[2];
        int n_want = 0;
        if (n_classes >= 3 && th != 2) want[n_want++] = 2;
        if (n_classes >= 2) want[n_want++] = th == 0 ? 1 : 0;
        if (n_want == 0) want[n_want++] = 0;
        const bool need_grad = !shared_grad || shared < 0;
        int c = take(want, n_want, need_grad ? 2 : 1);   // v_g and grad_g together
        if (c >= 0) {
            replicas[g].v = c;
            replicas[g].grad = need_grad ? c : shared;
        } else {
            if ((replicas[g].v = take(want, n_want, 1)) < 0) return full();
            replicas[g].grad = shared;
            if (need_grad && (replicas[g].grad = take(want, n_want, 1)) < 0) return full();
        }
        if (shared_grad && shared < 0) shared = replicas[g].grad;
    }
    return PIER_OK;
}

}  // extern "C"
