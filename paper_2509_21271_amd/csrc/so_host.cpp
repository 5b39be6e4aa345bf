// Host-only part of the C ABI (see include/so_adam.h): integer and scalar work that touches
// neither the GPU nor the HIP runtime -- the bucket layout planner, the arena layouts and the
// candidate placements of the placement search, the validation decision, the loss-scale
// schedule and the repartitioning inequality.  Kept in a plain C++ file so that
// it also builds with an ordinary host compiler (the sanitizer build of the CPU tests links
// exactly this file).
#include <cmath>
#include <cstddef>
#include <cstdint>

#include "../../include/so_adam.h"

extern "C" {

const char* so_version(void) { return "so_adam 0.2 (gfx950)"; }

// Bucketisation (Sec. 4.3): tensors back to back, cut every bucket_elems elements.
so_status so_layout_plan(const uint64_t* tensor_numel, size_t nt, uint64_t bucket_elems, so_slice* out,
                         size_t cap, size_t* n_slices, uint64_t* n_buckets)
{
    if ((!tensor_numel && nt) || bucket_elems == 0 || !n_slices || !n_buckets) return SO_ERR_INVALID_ARG;
    size_t count = 0;
    uint64_t flat = 0;   // running flat index
    for (size_t t = 0; t < nt; ++t) {
        uint64_t left = tensor_numel[t], toff = 0;
        while (left) {
            const uint64_t bk = flat / bucket_elems, boff = flat % bucket_elems;
            const uint64_t room = bucket_elems - boff;
            const uint64_t len = left < room ? left : room;
            if (out) {
                if (count >= cap) return SO_ERR_INVALID_ARG;
                out[count] = so_slice{(uint64_t)t, toff, bk, boff, len};
            }
            ++count;
            flat += len; toff += len; left -= len;
        }
    }
    *n_slices = count;
    *n_buckets = (flat + bucket_elems - 1) / bucket_elems;
    return SO_OK;
}

// Data layout in HBM: the five arenas of a model inside one allocation, order p g m q v, every
// arena on a 2 MiB boundary.
so_status so_arena_plan(uint64_t n_total, so_arena_layout* out)
{
    if (!out) return SO_ERR_INVALID_ARG;
    constexpr uint64_t kAlign = 2ull << 20;
    if (n_total > (~0ull - 8 * kAlign) / 16) return SO_ERR_INVALID_ARG;        // 16 n + slack must fit
    const uint64_t a4 = (n_total * 4 + kAlign - 1) / kAlign * kAlign;
    const uint64_t a2 = (n_total * 2 + kAlign - 1) / kAlign * kAlign;
    out->param = 0;
    out->grad = a4;
    out->exp_avg = a4 + a2;
    out->param_lp = 2 * a4 + a2;
    out->exp_avg_sq = 2 * a4 + 2 * a2;
    out->bytes = 3 * a4 + 2 * a2 + kAlign;
    return SO_OK;
}

// Candidate placements of so_arena_tune (see the header).
so_status so_arena_candidate(uint64_t n_total, uint64_t workspace_bytes, uint64_t seed, uint32_t index,
                             so_arena_layout* out, so_arena_alt* out_alt)
{
    so_arena_layout tight;
    if (!out || n_total == 0 || so_arena_plan(n_total, &tight) != SO_OK) return SO_ERR_INVALID_ARG;
    constexpr uint64_t kAlign = 2ull << 20;
    const int k = out_alt ? 9 : 5;
    const uint64_t a4 = tight.grad, a2 = tight.exp_avg - tight.grad;      // arena sizes rounded to 2 MiB
    // arena kinds in so_arena_plan's order p g m q v, then p' m' v' q'
    const uint64_t rounded[9] = {a4, a2, a4, a2, a4, a4, a4, a4, a2};
    const uint64_t bytes[9] = {n_total * 4, n_total * 2, n_total * 4, n_total * 2, n_total * 4,
                               n_total * 4, n_total * 4, n_total * 4, n_total * 2};
    uint64_t packed = 0;
    for (int a = 0; a < k; ++a) packed += rounded[a];
    if (workspace_bytes < packed) return SO_ERR_INVALID_ARG;      // every order must fit when packed
    const uint64_t slack = workspace_bytes > packed ? workspace_bytes - packed : 0;
    const uint64_t unit = slack / 256 / kAlign * kAlign;

    uint64_t state = seed ^ (0xD1B54A32D192ED03ull * ((uint64_t)index + 1));
    auto next = [&state]() {                      // splitmix64
        uint64_t z = (state += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    };
    int order[9];
    for (int a = 0; a < k; ++a) order[a] = a;
    uint64_t cuts[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
    if (index != 0) {
        for (int a = k - 1; a > 0; --a) {
            const int j = (int)(next() % (uint64_t)(a + 1));
            const int t = order[a]; order[a] = order[j]; order[j] = t;
        }
        if (unit != 0 && (index & 1u) == 0) {
            for (int a = 0; a < k; ++a) cuts[a] = next() % (slack / unit + 1);
            for (int a = 1; a < k; ++a)             // insertion sort: gaps are the differences
                for (int b = a; b > 0 && cuts[b - 1] > cuts[b]; --b) {
                    const uint64_t t = cuts[b]; cuts[b] = cuts[b - 1]; cuts[b - 1] = t;
                }
        }
    }
    uint64_t off[9], pos = 0, prev = 0, end = 0;
    for (int a = 0; a < k; ++a) {
        pos += (cuts[a] - prev) * unit;
        prev = cuts[a];
        off[order[a]] = pos;
        if (pos + bytes[order[a]] > end) end = pos + bytes[order[a]];
        pos += rounded[order[a]];
    }
    if (end > workspace_bytes) return SO_ERR_INVALID_ARG;      // cannot happen; kept as the last word
    out->param = off[0]; out->grad = off[1]; out->exp_avg = off[2]; out->param_lp = off[3];
    out->exp_avg_sq = off[4];
    out->bytes = end;
    if (out_alt) {
        out_alt->param = off[5]; out_alt->exp_avg = off[6]; out_alt->exp_avg_sq = off[7];
        out_alt->param_lp = off[8];
    }
    return SO_OK;
}

// Validation outcome (Sec. 4.4, the two rollback scenarios).
so_status so_validate(const so_stats* st, double max_norm, double loss_scale, double min_loss_scale, so_decision* out)
{
    if (!st || !out || !(loss_scale > 0.0)) return SO_ERR_INVALID_ARG;
    double clip = 1.0;
    if (max_norm > 0.0) {
        const double cc = max_norm / (st->norm + 1e-6);
        clip = cc < 1.0 ? cc : 1.0;
    }
    out->reserved = 0;
    out->clip = clip;
    out->grad_scale = (float)(clip / loss_scale);
    if (st->overflow) {
        const double half = loss_scale * 0.5;
        out->action = SO_ROLLBACK_SKIP;
        out->next_loss_scale = (float)(half > min_loss_scale ? half : min_loss_scale);
    } else {
        out->action = clip < 1.0 ? SO_ROLLBACK_REDO : SO_COMMIT;
        out->next_loss_scale = (float)loss_scale;
    }
    return SO_OK;
}

so_status so_loss_scale_next(float loss_scale, int overflow, uint32_t* clean_iterations, uint32_t growth_interval,
                             float min_loss_scale, float max_loss_scale, float* next_loss_scale)
{
    if (!clean_iterations || !next_loss_scale || !(loss_scale > 0.0f) || !(min_loss_scale > 0.0f) ||
        !(max_loss_scale >= min_loss_scale))
        return SO_ERR_INVALID_ARG;
    float next = loss_scale;
    if (overflow) {
        next = loss_scale * 0.5f;
        if (next < min_loss_scale) next = min_loss_scale;
        *clean_iterations = 0;
    } else {
        *clean_iterations += 1;
        if (growth_interval != 0 && *clean_iterations >= growth_interval) {
            next = loss_scale * 2.0f;
            if (next > max_loss_scale) next = max_loss_scale;
            *clean_iterations = 0;
        }
    }
    *next_loss_scale = next;
    return SO_OK;
}

// Bucket repartitioning (Sec. 4.3): smallest n with lhs <= n * per, capped.
so_status so_plan_resident(double move_grad_ms, double step_offloaded_ms, double move_param_ms,
                           double bwd_ms_per_bucket, double step_resident_ms_per_bucket,
                           uint64_t n_buckets, uint64_t max_resident, uint64_t* n_resident)
{
    if (!n_resident) return SO_ERR_INVALID_ARG;
    const double lhs = move_grad_ms + step_offloaded_ms + move_param_ms;
    const double per = bwd_ms_per_bucket + step_resident_ms_per_bucket;
    if (!(lhs >= 0.0) || !(per >= 0.0) || !std::isfinite(lhs) || !std::isfinite(per)) return SO_ERR_INVALID_ARG;
    const uint64_t cap = max_resident < n_buckets ? max_resident : n_buckets;
    uint64_t n = 0;
    while (n < cap && lhs > (double)n * per) ++n;
    *n_resident = n;
    return SO_OK;
}

}  // extern "C"
