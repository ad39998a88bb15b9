// Chunk-size selection across iterations by multiplicative increase, additive
// decrease (paper section 4.2.1).  A host-side state machine: the caller runs a
// collective with blink_miad_chunk(), measures its throughput, reports it, and
// repeats until blink_miad_steady().
//
// The paper gives the scheme in two sentences; the details fixed here: a
// measurement "increases" if it exceeds the previous one by more than rel_tol;
// the decrease phase keeps subtracting `step` while that raises the throughput
// and stops at the first step that does not; the steady chunk is the best one
// measured (the earlier one on a tie); bounds [lo, hi] end a phase when hit.
#include <cmath>
#include <new>

#include "../../include/blink.h"

struct blink_miad {
    enum Phase { kIncrease, kDecrease, kSteady };
    size_t chunk, step, lo, hi;
    double factor, rel_tol;
    Phase phase = kIncrease;
    bool have_prev = false, have_best = false;
    double prev = 0.0, best_throughput = 0.0;
    size_t best_chunk = 0;

    void settle() {
        phase = kSteady;
        chunk = best_chunk;
    }
    void shrink() {
        if (chunk < lo + step)
            settle();
        else
            chunk -= step;
    }
};

extern "C" {

blink_status_t blink_miad_create(size_t initial_chunk, double factor, size_t step, size_t lo,
                                 size_t hi, double rel_tol, blink_miad_t** out) {
    if (!out) return BLINK_EINVAL;
    *out = nullptr;
    if (initial_chunk < 1 || !(factor > 1.0) || !std::isfinite(factor) || step < 1 || lo < 1 ||
        hi < lo || !(rel_tol >= 0.0) || !std::isfinite(rel_tol))
        return BLINK_EINVAL;
    blink_miad* m = new (std::nothrow) blink_miad();
    if (!m) return BLINK_ENOMEM;
    m->chunk = initial_chunk < lo ? lo : (initial_chunk > hi ? hi : initial_chunk);
    m->step = step;
    m->lo = lo;
    m->hi = hi;
    m->factor = factor;
    m->rel_tol = rel_tol;
    *out = m;
    return BLINK_OK;
}

size_t blink_miad_chunk(const blink_miad_t* m) { return m ? m->chunk : 0; }
int blink_miad_steady(const blink_miad_t* m) { return m && m->phase == blink_miad::kSteady; }

blink_status_t blink_miad_report(blink_miad_t* m, double throughput) {
    if (!m || !std::isfinite(throughput) || throughput < 0.0) return BLINK_EINVAL;
    if (m->phase == blink_miad::kSteady) return BLINK_OK;
    if (!m->have_best || throughput > m->best_throughput) {
        m->have_best = true;
        m->best_throughput = throughput;
        m->best_chunk = m->chunk;
    }
    const bool rising = !m->have_prev || throughput > m->prev * (1.0 + m->rel_tol);
    m->have_prev = true;
    m->prev = throughput;
    if (m->phase == blink_miad::kIncrease) {
        if (rising) {
            const double grown = std::floor(static_cast<double>(m->chunk) * m->factor);
            const size_t next = grown >= static_cast<double>(m->hi) ? m->hi : static_cast<size_t>(grown);
            if (next == m->chunk)
                m->settle();
            else
                m->chunk = next;
        } else {
            m->phase = blink_miad::kDecrease;
            m->shrink();
        }
    } else if (rising) {
        m->shrink();
    } else {
        m->settle();
    }
    return BLINK_OK;
}

void blink_miad_free(blink_miad_t* m) { delete m; }

}  // extern "C"
