// Per-stage timing of the last dynbatch_execute / moe_forward call of this thread.
// Off by default; when on, an event is recorded after every launch group (execute) or stage (MoE).
#include "timing.h"

#include <vector>

#include "plan_internal.h"

namespace dynb {
namespace {

struct Mark {
    hipEvent_t ev;
    int32_t tag;
    int32_t units;
};

struct State {
    bool on = false;
    bool coarse = false;
    std::vector<hipEvent_t> pool;   // events are created once and reused
    std::vector<Mark> marks;        // marks[0] opens the call
    size_t used = 0;

    hipEvent_t next()
    {
        if (used == pool.size()) {
            hipEvent_t e = nullptr;
            if (hipEventCreate(&e) != hipSuccess) return nullptr;
            pool.push_back(e);
        }
        return pool[used++];
    }
};

thread_local State g;

}  // namespace

bool timing_on() { return g.on; }
bool timing_coarse() { return g.on && g.coarse; }

void timing_begin(hipStream_t st)
{
    g.marks.clear();
    g.used = 0;
    timing_mark(st, -1, 0);
}

void timing_mark(hipStream_t st, int32_t tag, int32_t units)
{
    hipEvent_t e = g.next();
    if (!e) return;
    if (hipEventRecord(e, st) != hipSuccess) return;
    g.marks.push_back(Mark{e, tag, units});
}

}  // namespace dynb

extern "C" int dynb_timing_enable(int on)
{
    if (on < 0 || on > 2) return dynb::fail(DYNB_E_INVAL, "dynb_timing_enable: mode must be 0, 1 or 2");
    dynb::g.on = (on != 0);
    dynb::g.coarse = (on == 2);
    return DYNB_OK;
}

extern "C" int dynb_timing_read(dynb_stage_time* out, int32_t capacity, int32_t* n_out)
{
    using namespace dynb;
    if (!n_out || (capacity > 0 && !out)) return fail(DYNB_E_INVAL, "dynb_timing_read: NULL argument");
    const int32_t n = g.marks.size() > 1 ? int32_t(g.marks.size() - 1) : 0;
    *n_out = n;
    if (n == 0) return DYNB_OK;
    hipError_t e = hipEventSynchronize(g.marks.back().ev);
    if (e != hipSuccess) return fail(DYNB_E_HIP, std::string("dynb_timing_read: ") + hipGetErrorString(e));
    for (int32_t i = 0; i < n && i < capacity; ++i) {
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, g.marks[i].ev, g.marks[i + 1].ev);
        if (e != hipSuccess) return fail(DYNB_E_HIP, std::string("dynb_timing_read: ") + hipGetErrorString(e));
        out[i].tag = g.marks[i + 1].tag;
        out[i].units = g.marks[i + 1].units;
        out[i].ms = ms;
    }
    return DYNB_OK;
}
