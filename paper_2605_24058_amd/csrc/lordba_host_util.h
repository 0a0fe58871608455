// Host helpers shared by the entry points of the LoRDBA library.
#pragma once
#include <hip/hip_runtime.h>

#include <mutex>

#include "lordba.h"

namespace {

// The kernels are built for gfx950 only; say so instead of failing inside the launch on another device.
lordba_status check_device() {
    static std::mutex mu;
    static int state[64] = {0};  // 0 unknown, 1 ok, 2 not usable
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return LORDBA_ERR_NO_DEVICE; }
    if (dev < 0 || dev >= 64) return LORDBA_ERR_NO_DEVICE;
    std::lock_guard<std::mutex> g(mu);
    if (state[dev] == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) { (void)hipGetLastError(); state[dev] = 2; }
        else {
            const char* n = prop.gcnArchName;
            bool ok = false;
            for (; n[0] && n[1] && n[2] && n[3] && n[4] && n[5]; ++n)
                if (n[0] == 'g' && n[1] == 'f' && n[2] == 'x' && n[3] == '9' && n[4] == '5' && n[5] == '0') { ok = true; break; }
            state[dev] = ok ? 1 : 2;
        }
    }
    return state[dev] == 1 ? LORDBA_OK : LORDBA_ERR_NO_DEVICE;
}

}  // namespace
