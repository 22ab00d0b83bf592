// Scope guard that makes one device current and puts the caller's device back on exit.
// The runtime calls come in through a policy type, so that the guard's logic can be exercised on a
// machine without a GPU (tests/host/device_guard_test.cpp instantiates it with a counting stand-in).
//   Api::get_device(int *out) -> bool, Api::set_device(int) -> bool, Api::clear_error().
#pragma once

namespace srs {

template <class Api>
struct BasicDeviceGuard {
    int prev = -1, target;
    bool ok;
    explicit BasicDeviceGuard(int device) : target(device) {
        ok = Api::get_device(&prev) && (prev == device || Api::set_device(device));
        if (!ok) Api::clear_error();
    }
    ~BasicDeviceGuard() {
        // one plain call: the caller's device goes back exactly once, whatever it was
        if (ok && prev != target && !Api::set_device(prev)) Api::clear_error();
    }
    BasicDeviceGuard(const BasicDeviceGuard &) = delete;
    BasicDeviceGuard &operator=(const BasicDeviceGuard &) = delete;
};

}  // namespace srs
