// Host-only check of the device guard: a counting stand-in replaces the GPU runtime.
// Prints one line per scenario; exit status 0 when every expectation holds.
#include "device_guard.hpp"

#include <cstdio>

namespace {
int g_current = 0, g_gets = 0, g_sets = 0, g_clears = 0, g_fail_set_to = -1;

struct MockApi {
    static bool get_device(int *out) { ++g_gets; *out = g_current; return true; }
    static bool set_device(int d) {
        ++g_sets;
        if (d == g_fail_set_to) return false;
        g_current = d;
        return true;
    }
    static void clear_error() { ++g_clears; }
};
typedef srs::BasicDeviceGuard<MockApi> Guard;

void reset(int current) { g_current = current; g_gets = g_sets = g_clears = 0; g_fail_set_to = -1; }

int check(const char *what, bool cond) {
    std::printf("%s: %s\n", what, cond ? "ok" : "FAILED");
    return cond ? 0 : 1;
}
}  // namespace

int main() {
    int bad = 0;
    reset(0);
    { Guard g(0); bad += check("same device: usable", g.ok && g_current == 0); }
    bad += check("same device: no switch at all", g_sets == 0 && g_gets == 1 && g_current == 0);

    reset(3);
    {
        Guard g(1);
        bad += check("other device: target is current inside the scope", g.ok && g_current == 1 && g_sets == 1);
    }
    bad += check("other device: caller's device restored by exactly one more call", g_current == 3 && g_sets == 2);

    reset(2);
    {
        Guard outer(0);
        { Guard inner(5); bad += check("nested: inner target current", g_current == 5); }
        bad += check("nested: back to the outer target", g_current == 0);
    }
    bad += check("nested: back to the caller's device", g_current == 2 && g_sets == 4);

    reset(4);
    g_fail_set_to = 1;
    {
        Guard g(1);
        bad += check("switch fails: guard reports it, device untouched", !g.ok && g_current == 4 && g_clears == 1);
    }
    bad += check("switch fails: destructor does nothing", g_current == 4 && g_sets == 1);
    return bad ? 1 : 0;
}
