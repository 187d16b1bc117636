// Variable batch size per layer (Sec. V-C, "Dynamic Programming").
//
// OPT(i, B, A): least time to run layers 1..i when layer i uses batch B and A
// units of memory are held back for the later layers.  With layer i-1 at batch b
// (b divides B) the earlier layers run B / b times, and before the last of those
// runs IN(i, B - b) of layer i's input is already parked, so
//     OPT(i, B, A) = Time(i, B) + min_b (B / b) * OPT(i-1, b, A + IN(i, B - b))
// subject to A + IN(i,B) + WS(i) + OUT(i,B) <= TOT; an entry above the latency
// threshold is infinite.  The answer is min_B OPT(f, B, 0) / B.
//
// Only states reachable from <f, B, 0> are evaluated (memoised recursion), so the
// reserved-memory axis may be as fine as the caller likes.
#include <cmath>
#include <limits>
#include <map>
#include <tuple>
#include <vector>

#include "layer.hpp"

namespace {

struct Planner {
    int f, nb;
    const int32_t *bs;
    const double *time_ms;
    const int64_t *inb, *outb, *ws;
    int64_t tot, step;
    double cap;
    struct Cell { double t; int prev_j; };
    std::map<std::tuple<int, int, int64_t>, Cell> memo;

    static int64_t units(int64_t bytes, int64_t step) { return (bytes + step - 1) / step; }

    Cell opt(int i, int j, int64_t A)
    {
        const auto key = std::make_tuple(i, j, A);
        auto it = memo.find(key);
        if (it != memo.end()) return it->second;
        const double inf = std::numeric_limits<double>::infinity();
        Cell cell{inf, -1};
        const int64_t B = bs[j];
        if (A * step + B * inb[i] + ws[i] + B * outb[i] <= tot) {
            const double t = time_ms[(size_t)i * nb + j];
            if (i == 0) {
                if (t <= cap) cell.t = t;
            } else {
                double best = inf;
                int arg = -1;
                for (int jj = 0; jj < nb; ++jj) {
                    const int64_t b = bs[jj];
                    if (b > B || B % b) continue;
                    const Cell sub = opt(i - 1, jj, units(A * step + (B - b) * inb[i], step));
                    if (std::isinf(sub.t)) continue;
                    const double c = (double)(B / b) * sub.t;
                    if (c < best) { best = c; arg = jj; }
                }
                if (arg >= 0 && t + best <= cap) { cell.t = t + best; cell.prev_j = arg; }
            }
        }
        memo.emplace(key, cell);
        return cell;
    }
};

}  // namespace

extern "C" int32_t cl_plan_batches(int32_t n_layers, const int32_t *batch_set, int32_t n_batches,
                                   const double *time_ms, const int64_t *in_bytes_per_image,
                                   const int64_t *out_bytes_per_image, const int64_t *ws_bytes,
                                   int64_t tot_bytes, int64_t mem_step_bytes, double latency_cap_ms,
                                   int32_t *out_batch_per_layer, double *out_ms_per_image)
{
    using cl::fail;
    if (!batch_set || !time_ms || !in_bytes_per_image || !out_bytes_per_image || !ws_bytes || !out_batch_per_layer || !out_ms_per_image)
        return fail(CL_EINVAL, "null argument");
    if (n_layers < 1 || n_batches < 1 || mem_step_bytes < 1 || tot_bytes < 0) return fail(CL_EINVAL, "bad sizes");
    for (int j = 0; j < n_batches; ++j)
        if (batch_set[j] < 1 || (j && batch_set[j] <= batch_set[j - 1])) return fail(CL_EINVAL, "batch_set must be positive and ascending");
    for (int i = 0; i < n_layers; ++i) {
        if (in_bytes_per_image[i] < 0 || out_bytes_per_image[i] < 0 || ws_bytes[i] < 0) return fail(CL_EINVAL, "negative memory size");
        for (int j = 0; j < n_batches; ++j) {
            const double t = time_ms[(size_t)i * n_batches + j];
            if (!(t >= 0.0) || std::isinf(t)) return fail(CL_EINVAL, "Time(%d,%d) is not a finite non-negative number", i, batch_set[j]);
        }
    }
    Planner P{n_layers, n_batches, batch_set, time_ms, in_bytes_per_image, out_bytes_per_image, ws_bytes,
              tot_bytes, mem_step_bytes, latency_cap_ms > 0 ? latency_cap_ms : std::numeric_limits<double>::infinity(), {}};
    double best = std::numeric_limits<double>::infinity();
    int arg = -1;
    for (int j = 0; j < n_batches; ++j) {
        const auto cell = P.opt(n_layers - 1, j, 0);
        if (std::isinf(cell.t)) continue;
        const double per = cell.t / (double)batch_set[j];
        if (per < best) { best = per; arg = j; }
    }
    *out_ms_per_image = best;
    if (arg < 0) {
        for (int i = 0; i < n_layers; ++i) out_batch_per_layer[i] = 0;
        return fail(CL_EUNSUPPORTED, "no feasible plan under the memory and latency limits");
    }
    // walk the chosen chain back
    int j = arg;
    int64_t A = 0;
    for (int i = n_layers - 1; i >= 0; --i) {
        out_batch_per_layer[i] = batch_set[j];
        if (i == 0) break;
        const auto cell = P.opt(i, j, A);
        const int64_t B = batch_set[j], b = batch_set[cell.prev_j];
        A = Planner::units(A * mem_step_bytes + (B - b) * in_bytes_per_image[i], mem_step_bytes);
        j = cell.prev_j;
    }
    cl::clear_error();
    return CL_OK;
}
