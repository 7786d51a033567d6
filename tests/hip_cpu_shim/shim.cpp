// Runtime of the host stand-in for HIP (see hip/hip_runtime.h).  Test infrastructure only.
#include <hip/hip_runtime.h>

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
// the threads of the workgroup that is running (a launch runs its workgroups in turn)
struct Team {
    std::unique_ptr<std::barrier<>> bar;
    std::vector<uint32_t> exchange;
    int lanes = 0;
};
Team team;
thread_local bool left_team = false;
int last_error = hipSuccess;
}  // namespace

void barrier_wait() { team.bar->arrive_and_wait(); }

uint32_t shuffle_xor(uint32_t v, int mask)
{
    const int lane = (int)threadIdx.x;
    team.exchange[lane] = v;
    team.bar->arrive_and_wait();
    const int src = lane ^ mask;
    const uint32_t got = src < team.lanes ? team.exchange[src] : v;
    team.bar->arrive_and_wait();
    return got;
}

void launch(dim3 grid, dim3 block, size_t lds, const std::function<void()> &body)
{
    launches++;
    if (grid.x == 0 || block.x == 0 || block.x > 1024 || lds > max_dynamic_lds) {
        std::fprintf(stderr, "shim: launch refused (grid %u, block %u, lds %zu)\n", grid.x, block.x, lds);
        last_error = hipErrorInvalidValue;
        return;
    }
    // One thread per lane, kept for the whole launch; the workgroups run one after the other.
    // team.bar serves __syncthreads() inside a workgroup (a lane that has returned drops out
    // of it); between_blocks keeps the lanes together from one workgroup to the next.
    const int n = (int)block.x;
    std::barrier<> between_blocks(n);
    unsigned char *smem = nullptr;
    auto new_block = [&] {
        std::free(smem);
        smem = lds ? static_cast<unsigned char *>(std::malloc(lds)) : nullptr;
        team.bar = std::make_unique<std::barrier<>>(n);
    };
    team.exchange.assign(n, 0);
    team.lanes = n;
    new_block();
    std::vector<std::thread> pool;
    pool.reserve(n);
    for (int t = 0; t < n; t++)
        pool.emplace_back([&, t] {
            blockDim = block;
            gridDim = grid;
            for (unsigned b = 0; b < grid.x; b++) {
                threadIdx = {(unsigned)t, 0, 0};
                blockIdx = {b, 0, 0};
                dyn_smem = smem;
                body();
                team.bar->arrive_and_drop();            // a lane that is done no longer holds up the others
                between_blocks.arrive_and_wait();
                if (t == 0 && b + 1 < grid.x) new_block();
                between_blocks.arrive_and_wait();
            }
        });
    for (auto &th : pool) th.join();
    std::free(smem);
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
