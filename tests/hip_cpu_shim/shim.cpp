// Runtime of the host stand-in for HIP (see hip/hip_runtime.h).  Test infrastructure only.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>

thread_local shim_uint3 threadIdx, blockIdx;
thread_local dim3 blockDim, gridDim;

namespace shim {
thread_local unsigned char *dyn_smem = nullptr;
int compute_units = 8;
int blocks_per_cu = 4;
size_t max_dynamic_lds = 64 * 1024;
std::atomic<long> launches{0};

namespace {
// State of one workgroup of the running launch.  The lanes (one OS thread each, kept for the
// whole launch) walk the workgroups in order but NOT in step: a lane only waits for the other
// lanes of its workgroup where the kernel itself synchronises (__syncthreads, lane shuffles), so
// kernels without barriers cost no system calls per workgroup.  A lane that has returned from
// the kernel counts as arrived at every later barrier of that workgroup.
struct Block {
    std::mutex m;
    std::condition_variable cv;
    int waiting = 0, done = 0;
    unsigned long generation = 0;
    unsigned char *smem = nullptr;        // dynamic LDS, made by the first lane that gets here
    void *statics = nullptr;              // the kernel's static __shared__ array, if it has one
    std::vector<uint32_t> exchange;       // lane shuffles
};
struct Launch {
    std::unique_ptr<Block[]> blocks;
    int lanes = 0;
    size_t lds = 0;
};
Launch cur;
thread_local Block *my_block = nullptr;
int last_error = hipSuccess;
constexpr unsigned kWindow = 32;          // a lane runs at most this many workgroups ahead of the slowest
}  // namespace

void barrier_wait()
{
    Block &b = *my_block;
    std::unique_lock<std::mutex> lock(b.m);
    if (++b.waiting + b.done == cur.lanes) {
        b.waiting = 0;
        b.generation++;
        b.cv.notify_all();
    } else {
        const unsigned long g = b.generation;
        b.cv.wait(lock, [&] { return b.generation != g; });
    }
}

uint32_t shuffle_xor(uint32_t v, int mask)
{
    Block &b = *my_block;
    const int lane = (int)threadIdx.x;
    {
        std::lock_guard<std::mutex> lock(b.m);
        if (b.exchange.empty()) b.exchange.assign(cur.lanes, 0);
        b.exchange[lane] = v;
    }
    barrier_wait();
    const int src = lane ^ mask;
    uint32_t got = v;
    {
        std::lock_guard<std::mutex> lock(b.m);
        if (src < cur.lanes) got = b.exchange[src];
    }
    barrier_wait();
    return got;
}

void *block_static(size_t bytes)
{
    Block &b = *my_block;
    std::lock_guard<std::mutex> lock(b.m);
    if (!b.statics) b.statics = std::malloc(bytes);
    return b.statics;
}

void launch(dim3 grid, dim3 block, size_t lds, const std::function<void()> &body)
{
    launches++;
    if (grid.x == 0 || block.x == 0 || block.x > 1024 || lds > max_dynamic_lds) {
        std::fprintf(stderr, "shim: launch refused (grid %u, block %u, lds %zu)\n", grid.x, block.x, lds);
        last_error = hipErrorInvalidValue;
        return;
    }
    const int n = (int)block.x;
    cur.blocks.reset(new Block[grid.x]);
    cur.lanes = n;
    cur.lds = lds;
    std::vector<std::atomic<unsigned>> progress(n);
    for (auto &p : progress) p.store(0);
    std::vector<std::thread> pool;
    pool.reserve(n);
    for (int t = 0; t < n; t++)
        pool.emplace_back([&, t] {
            blockDim = block;
            gridDim = grid;
            for (unsigned b = 0; b < grid.x; b++) {
                if (b >= kWindow && b % 8 == 0) {       // bound the memory of workgroups in progress
                    for (;;) {
                        unsigned slowest = b;
                        for (auto &p : progress) slowest = std::min(slowest, p.load(std::memory_order_relaxed));
                        if (slowest + kWindow > b) break;
                        std::this_thread::yield();
                    }
                }
                Block &blk = cur.blocks[b];
                my_block = &blk;
                threadIdx = {(unsigned)t, 0, 0};
                blockIdx = {b, 0, 0};
                dyn_smem = nullptr;
                if (lds) {
                    std::lock_guard<std::mutex> lock(blk.m);
                    if (!blk.smem) blk.smem = static_cast<unsigned char *>(std::malloc(lds));
                    dyn_smem = blk.smem;
                }
                body();
                {
                    std::lock_guard<std::mutex> lock(blk.m);
                    if (++blk.done == n) {                // last lane out frees the workgroup's memory
                        std::free(blk.smem);
                        std::free(blk.statics);
                        blk.smem = nullptr;
                        blk.statics = nullptr;
                    } else if (blk.waiting > 0 && blk.waiting + blk.done == n) {
                        blk.waiting = 0;                  // the others were waiting for this lane only
                        blk.generation++;
                        blk.cv.notify_all();
                    }
                }
                progress[t].store(b + 1, std::memory_order_relaxed);
            }
        });
    for (auto &th : pool) th.join();
    cur.blocks.reset();
}
}  // namespace shim

hipError_t hipMalloc(void **p, size_t bytes)
{
    *p = std::malloc(bytes ? bytes : 1);
    return *p ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipFree(void *p) { std::free(p); return hipSuccess; }
hipError_t hipMemcpy(void *dst, const void *src, size_t bytes, hipMemcpyKind) { std::memcpy(dst, src, bytes); return hipSuccess; }
hipError_t hipGetDevice(int *dev) { *dev = 0; return hipSuccess; }
hipError_t hipSetDevice(int) { return hipSuccess; }
hipError_t hipGetLastError() { const int e = shim::last_error; shim::last_error = hipSuccess; return e; }
hipError_t hipDeviceGetAttribute(int *out, hipDeviceAttribute_t, int) { *out = shim::compute_units; return hipSuccess; }
hipError_t hipEventCreateWithFlags(hipEvent_t *ev, unsigned) { *ev = reinterpret_cast<hipEvent_t>(std::malloc(1)); return hipSuccess; }
hipError_t hipEventDestroy(hipEvent_t ev) { std::free(ev); return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t, unsigned) { return hipSuccess; }
hipError_t hipStreamIsCapturing(hipStream_t, hipStreamCaptureStatus *out) { *out = hipStreamCaptureStatusNone; return hipSuccess; }
hipError_t hipGetSymbolAddress(void **out, const void *symbol) { *out = const_cast<void *>(symbol); return hipSuccess; }
