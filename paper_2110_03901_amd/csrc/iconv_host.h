// Host-side helpers shared by the launchers of the persistent kernels.
#pragma once
#include <atomic>

#include "iconv_common.h"

namespace iconv {

// Number of compute units of the current device (cached).
inline int device_cus() {
    static std::atomic<int> cus{0};
    int v = cus.load(std::memory_order_acquire);
    if (v == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1)
            v = 256;
        cus.store(v, std::memory_order_release);
    }
    return v;
}

// Splits `total` tiles over workgroups: k resident workgroups per compute unit for k = 1..occ,
// each owning ceil(total / (cus*k)) contiguous tiles; takes the k with the fewest tiles on the
// busiest compute unit, the larger k on a tie (more independent workgroups to overlap).
inline void split_tiles(long total, int cus, int occ, int* per_wg, int* nwg) {
    long best_load = -1;
    for (int k = 1; k <= occ; ++k) {
        const long per = (total + (long)cus * k - 1) / ((long)cus * k);
        const long n = (total + per - 1) / per;
        const long load = per * ((n + cus - 1) / cus);
        if (best_load < 0 || load <= best_load) {
            best_load = load;
            *per_wg = (int)per;
            *nwg = (int)n;
        }
    }
}

// Resident workgroups per compute unit of `kern` at `lds_bytes` of dynamic LDS, cached per call
// site in `slot` (initialise it to -1): LDS size and result travel in ONE atomic word, so concurrent
// callers with different sizes never pair one's size with the other's result.
inline int cached_occupancy(std::atomic<long long>& slot, const void* kern, int threads, int lds_bytes) {
    const long long cur = slot.load(std::memory_order_acquire);
    if (cur >= 0 && (int)(cur >> 8) == lds_bytes) return (int)(cur & 0xff);
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kern, threads, (size_t)lds_bytes) != hipSuccess || nb < 1) nb = 1;
    if (nb > 255) nb = 255;
    slot.store(((long long)lds_bytes << 8) | nb, std::memory_order_release);
    return nb;
}

// Cap on the number of workgroups of a persistent launch asked for by the call that is running on
// this thread (0 = none; only iconv_fwd_ex sets one, for its own duration).
int call_max_workgroups();

}  // namespace iconv
