// Host-side recommendation of a mixed-precision setting: the Accuracy-Decay-Aware allocator
// (Section 3.2, Algorithm 1) and the threshold rules of Appendix A.  Pure host code: the inputs are
// the per-setting accuracies (from the caller's evaluation) and latencies (measured with this
// library's encoder), setting 0 being all-FP16 and later settings quantising more layers.
#include "samp_common.h"

#include <algorithm>
#include <cmath>
#include <limits>

namespace samp {

// Algorithm 1.  The recommended setting moves to i whenever the accuracy change per latency change
// since the last recommended setting, dr, is negative or below every rate accepted so far.
// A zero latency difference is resolved by the sign of the accuracy difference (gain: accepted,
// loss: rejected, none: skipped).
int allocate_decay_aware(const double *A, const double *L, int n)
{
    int rec = 0;
    double dr_min = std::numeric_limits<double>::infinity();
    for (int i = 1; i < n; i++) {
        const double da = A[i] - A[rec], dl = L[i] - L[rec];
        double dr;
        if (dl != 0.0) dr = da / dl;
        else if (da > 0.0) dr = -std::numeric_limits<double>::infinity();
        else if (da < 0.0) dr = std::numeric_limits<double>::infinity();
        else continue;
        if (dr < 0.0 || dr < dr_min) {
            dr_min = dr;
            rec = i;
        }
    }
    return rec;
}

// Appendix A.  max_latency set (not NaN): the most accurate setting no slower than it.  Otherwise
// min_accuracy set: the fastest setting no less accurate than it.  Otherwise up to five settings
// i >= 1 in decreasing order of speedup over accuracy loss, (L[0] / L[i]) / (A[0] - A[i]); settings
// without a loss rank first, by speedup.  Ties keep the setting with fewer quantised layers.
// Returns the number of settings written to out (at most cap).
int recommend_settings(const double *A, const double *L, int n, double max_latency, double min_accuracy, int *out, int cap)
{
    if (cap < 1) return 0;
    if (!std::isnan(max_latency)) {
        int best = -1;
        for (int i = 0; i < n; i++)
            if (L[i] <= max_latency && (best < 0 || A[i] > A[best])) best = i;
        if (best < 0) return 0;
        out[0] = best;
        return 1;
    }
    if (!std::isnan(min_accuracy)) {
        int best = -1;
        for (int i = 0; i < n; i++)
            if (A[i] >= min_accuracy && (best < 0 || L[i] < L[best])) best = i;
        if (best < 0) return 0;
        out[0] = best;
        return 1;
    }
    struct Cand { bool lossy; double score; int i; };
    Cand cand[64];
    int nc = 0;
    for (int i = 1; i < n && nc < 64; i++) {
        const double speedup = L[0] / L[i], loss = A[0] - A[i];
        cand[nc++] = loss > 0.0 ? Cand{true, speedup / loss, i} : Cand{false, speedup, i};
    }
    std::stable_sort(cand, cand + nc, [](const Cand &a, const Cand &b) {
        if (a.lossy != b.lossy) return !a.lossy;
        return a.score > b.score;
    });
    const int take = std::min(std::min(nc, 5), cap);
    for (int k = 0; k < take; k++) out[k] = cand[k].i;
    return take;
}

}  // namespace samp
