// Per-device host state shared by the launchers: the compute-unit count of each device, read once.
#include "fq_kernels.h"

int fq_current_device_slot() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    return (dev >= 0 && dev < FQ_MAX_DEVICES) ? dev : 0;
}

int fq_device_cus() {
    static std::atomic<int> cus[FQ_MAX_DEVICES];           // 0 = not read yet
    const int d = fq_current_device_slot();
    int v = cus[d].load(std::memory_order_relaxed);
    if (v > 0) return v;
    int dev = 0;
    v = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) {
        (void)hipGetLastError();
        v = 256;
    }
    cus[d].store(v, std::memory_order_relaxed);
    return v;
}
