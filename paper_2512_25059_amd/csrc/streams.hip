// Library-owned side streams for the fork/join inside one call (see ForkJoin in r2_internal.h).
#include <mutex>

#include "r2_internal.h"

namespace r2 {

struct Pool {
    std::mutex issue;  // one forking call at a time per device: the events are shared
    bool ready = false;
    hipStream_t side[kSideStreams] = {};
    hipEvent_t fork = nullptr, done[kSideStreams] = {};
};

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_lock;
Pool g_pools[kMaxDevices];

// The pool of the current device, created on first use; null if the runtime refuses.
Pool *pool_of_current_device()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> hold(g_lock);
    Pool &p = g_pools[dev];
    if (p.ready) return &p;
    // default priority: streams of different priorities are not mixed
    if (hipEventCreateWithFlags(&p.fork, hipEventDisableTiming) != hipSuccess) return nullptr;
    for (unsigned i = 0; i < kSideStreams; ++i) {
        if (hipStreamCreateWithFlags(&p.side[i], hipStreamNonBlocking) != hipSuccess) return nullptr;
        if (hipEventCreateWithFlags(&p.done[i], hipEventDisableTiming) != hipSuccess) return nullptr;
    }
    p.ready = true;
    return &p;
}

}  // namespace

ForkJoin::ForkJoin(hipStream_t user) : user_(user), pool_(pool_of_current_device())
{
    if (!pool_) {
        rc_ = R2_ERR_DEVICE;
        return;
    }
    pool_->issue.lock();
    // The fork point is where the call starts: work it puts on the caller's stream afterwards must
    // not hold the other lanes back.
    if (hipEventRecord(pool_->fork, user_) != hipSuccess) rc_ = R2_ERR_DEVICE;
}

ForkJoin::~ForkJoin()
{
    if (!pool_) return;
    (void)join();  // a call that returns early still leaves the caller's stream behind every lane
    pool_->issue.unlock();
}

hipStream_t ForkJoin::lane(unsigned i)
{
    if (i == 0 || rc_ != R2_OK) return user_;
    const unsigned k = (i - 1) % kSideStreams;
    if (!used_[k]) {
        if (hipStreamWaitEvent(pool_->side[k], pool_->fork, 0) != hipSuccess) rc_ = R2_ERR_DEVICE;
        used_[k] = true;
    }
    return rc_ == R2_OK ? pool_->side[k] : user_;
}

int ForkJoin::join()
{
    for (unsigned k = 0; k < kSideStreams && rc_ == R2_OK; ++k) {
        if (!used_[k]) continue;
        if (hipEventRecord(pool_->done[k], pool_->side[k]) != hipSuccess ||
            hipStreamWaitEvent(user_, pool_->done[k], 0) != hipSuccess)
            rc_ = R2_ERR_DEVICE;
        used_[k] = false;
    }
    return rc_;
}

}  // namespace r2
