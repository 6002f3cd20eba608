// Shuffle Scheduler rate rule (Sec. 5, Eq. 5).  Host-only state machine: the caller reports
// the test loss after every swap between cold and hot mini-batches and gets the rate R(p)
// to use next.  The clamps follow the text of Sec. 5 (never below R(1), never above R(100));
// the printed equation has min and max the other way round.
#include "fae_internal.h"

#include <math.h>

extern "C" int32_t fae_sched_init(fae_sched *s, double p0, int32_t u)
{
    if (!s || !(p0 >= 1.0 && p0 <= 100.0) || u < 1)
        return FAE_EINVAL;
    s->rate = p0;
    s->prev = 0.0;
    s->u = u;
    s->falls = 0;
    s->reports = 0;
    return FAE_OK;
}

extern "C" double fae_sched_report(fae_sched *s, double test_loss)
{
    if (!s || s->u < 1 || test_loss != test_loss)
        return -1.0;
    if (s->reports > 0) {
        if (test_loss >= s->prev) { // the loss did not fall: shuffle more often
            s->rate = s->rate * 0.5 < 1.0 ? 1.0 : s->rate * 0.5;
            s->falls = 0;
        } else if (++s->falls >= s->u) { // u falls in a row: shuffle less often
            s->rate = s->rate * 2.0 > 100.0 ? 100.0 : s->rate * 2.0;
            s->falls = 0;
        }
    }
    s->prev = test_loss;
    s->reports += 1;
    return s->rate;
}

extern "C" int64_t fae_sched_segment(const fae_sched *s, int64_t n_total)
{
    if (!s || n_total <= 0)
        return 0;
    const int64_t seg = (int64_t)ceil(s->rate / 100.0 * (double)n_total);
    return seg < 1 ? 1 : (seg > n_total ? n_total : seg);
}
