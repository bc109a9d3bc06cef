// Depth schedule and layer-index table of D^3 (pure host code, no GPU).
//
// Section 3.4 gives the number of blocks kept when generating token T_i as
// floor(L * alpha^i); Table 6 gives the dropped blocks as a contiguous window of
// middle blocks that begins at `start` and grows with i.  Readings fixed here:
//   * alpha^i is built by repeated binary64 multiplication, so the table is the same on
//     every IEEE-754 host, whatever its libm;
//   * exactly keep[i] blocks run: the window is [s_i, s_i + n_i) with n_i = L - keep[i];
//   * when the window would run past the last block it is shifted down,
//     s_i = min(start, L - n_i), which keeps the count exact and the windows nested.
#include <cmath>
#include <cstdint>

#include "../../include/d3.h"
#include "d3_error.h"

namespace {

// Window and executed-block list of one step that keeps `kept` of L blocks.
void emit_step(int32_t L, int32_t start_layer, int32_t i, int32_t kept, int32_t* keep, int32_t* drop_begin, int32_t* layer_ids) {
    const int32_t n_drop = L - kept;
    const int32_t first = start_layer + n_drop <= L ? start_layer : L - n_drop;
    if (keep) keep[i] = kept;
    if (drop_begin) drop_begin[i] = first;
    if (layer_ids) {
        int32_t* ids = layer_ids + static_cast<size_t>(i) * L;
        int32_t j = 0;
        for (int32_t l = 0; l < first; ++l) ids[j++] = l;
        for (int32_t l = first + n_drop; l < L; ++l) ids[j++] = l;
        while (j < L) ids[j++] = -1;
    }
}

}  // namespace

extern "C" int d3_plan_depth(int32_t L, double alpha, int32_t start_layer, int32_t min_keep, int32_t n_steps,
                             int32_t* keep, int32_t* drop_begin, int32_t* layer_ids) {
    if (L < 1) return d3::fail(D3_EINVAL, "d3_plan_depth: L must be >= 1 (got %d)", L);
    if (!(alpha > 0.0 && alpha <= 1.0)) return d3::fail(D3_EINVAL, "d3_plan_depth: alpha must be in (0, 1] (got %g)", alpha);
    if (start_layer < 0 || start_layer >= L)
        return d3::fail(D3_EINVAL, "d3_plan_depth: start_layer must be in [0, %d) (got %d)", L, start_layer);
    if (min_keep < 0 || min_keep > L) return d3::fail(D3_EINVAL, "d3_plan_depth: min_keep must be in [0, %d] (got %d)", L, min_keep);
    if (n_steps < 0) return d3::fail(D3_EINVAL, "d3_plan_depth: n_steps must be >= 0 (got %d)", n_steps);

    double decay = 1.0;                               // alpha^i
    for (int32_t i = 0; i < n_steps; ++i, decay *= alpha) {
        int32_t kept = static_cast<int32_t>(std::floor(static_cast<double>(L) * decay));
        if (kept < min_keep) kept = min_keep;
        emit_step(L, start_layer, i, kept, keep, drop_begin, layer_ids);
    }
    return D3_OK;
}

// Linear decay between two bounds (the comparison schedule that Section 3.4 and Section 4.1 set against the power
// law): keep[i] = floor(keep_first - (keep_first - keep_last) * i / (n_steps - 1)), in integers.  The same window
// rule places the dropped blocks, so start_layer = 0 drops the shallow blocks first and start_layer = L - 1 the
// deep ones (the two directions of Section 1's comparison).
extern "C" int d3_plan_depth_linear(int32_t L, int32_t keep_first, int32_t keep_last, int32_t start_layer, int32_t n_steps,
                                    int32_t* keep, int32_t* drop_begin, int32_t* layer_ids) {
    if (L < 1) return d3::fail(D3_EINVAL, "d3_plan_depth_linear: L must be >= 1 (got %d)", L);
    if (keep_last < 0 || keep_last > keep_first || keep_first > L)
        return d3::fail(D3_EINVAL, "d3_plan_depth_linear: need 0 <= keep_last <= keep_first <= L (got %d, %d, L = %d)", keep_last, keep_first, L);
    if (start_layer < 0 || start_layer >= L)
        return d3::fail(D3_EINVAL, "d3_plan_depth_linear: start_layer must be in [0, %d) (got %d)", L, start_layer);
    if (n_steps < 0) return d3::fail(D3_EINVAL, "d3_plan_depth_linear: n_steps must be >= 0 (got %d)", n_steps);

    const int64_t span = keep_first - keep_last, last = n_steps > 1 ? n_steps - 1 : 1;
    for (int32_t i = 0; i < n_steps; ++i) {
        const int64_t lost = (span * i + last - 1) / last;          // ceil(span * i / last)
        emit_step(L, start_layer, i, static_cast<int32_t>(keep_first - lost), keep, drop_begin, layer_ids);
    }
    return D3_OK;
}

// Executed-block lists of a schedule the caller made: validates every step and writes its list.
extern "C" int d3_plan_from_table(int32_t L, int32_t n_steps, const int32_t* keep, const int32_t* drop_begin, int32_t* layer_ids) {
    if (L < 1 || n_steps < 0 || (n_steps > 0 && (!keep || !drop_begin)))
        return d3::fail(D3_EINVAL, "d3_plan_from_table: need L >= 1, n_steps >= 0 and both tables");
    for (int32_t i = 0; i < n_steps; ++i) {
        const int32_t n_drop = L - keep[i];
        if (keep[i] < 0 || keep[i] > L || drop_begin[i] < 0 || drop_begin[i] + n_drop > L || (n_drop > 0 && drop_begin[i] >= L))
            return d3::fail(D3_EINVAL, "d3_plan_from_table: step %d keeps %d of %d blocks with a window at %d", i, keep[i], L, drop_begin[i]);
        if (layer_ids) emit_step(L, drop_begin[i], i, keep[i], nullptr, nullptr, layer_ids);
    }
    return D3_OK;
}
