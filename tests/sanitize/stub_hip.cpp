// A HIP runtime made of host code only, for running the executor's issue logic under ThreadSanitizer without a GPU.
// Streams are opaque handles that are never dereferenced; an event counts its records; nothing executes.  What the stub
// checks is the one rule the executor's per-tenant issue threads must keep (a hipStreamWaitEvent only sees records that
// were issued before it): for every (event, waiting stream) pair it learns, from rounds issued by a single thread, how
// many waits a round holds, and afterwards requires that the n-th wait of the pair finds at least n / that + 1 records.
#include <hip/hip_runtime_api.h>
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>

namespace {
struct Ev {
    std::atomic<long> records{0};
    long rec_base = 0;
    std::mutex mu;
    std::map<const void *, long> waits, wait_base, per_round;      // by waiting stream
};
std::atomic<long> g_violations{0}, g_waits_checked{0};
std::atomic<int> g_phase{0};           // 0 idle, 1 learning (single thread), 2 checking
std::mutex g_all_mu;
std::map<Ev *, int> g_all;
}  // namespace

extern "C" {
void stub_learn_begin() { g_phase = 1; std::lock_guard<std::mutex> g(g_all_mu); for (auto &kv : g_all) { Ev *e = kv.first; e->rec_base = e->records; e->wait_base = e->waits; } }
void stub_learn_end(int rounds)
{
    std::lock_guard<std::mutex> g(g_all_mu);
    for (auto &kv : g_all) {
        Ev *e = kv.first;
        e->per_round.clear();
        for (auto &w : e->waits) e->per_round[w.first] = (w.second - e->wait_base[w.first]) / rounds;
    }
    g_phase = 0;
}
void stub_check_begin() { std::lock_guard<std::mutex> g(g_all_mu); for (auto &kv : g_all) { Ev *e = kv.first; e->rec_base = e->records; e->wait_base = e->waits; } g_phase = 2; }
void stub_check_end() { g_phase = 0; }
long stub_violations() { return g_violations; }
long stub_waits_checked() { return g_waits_checked; }

hipError_t hipGetDevice(int *d) { *d = 0; return hipSuccess; }
hipError_t hipSetDevice(int) { return hipSuccess; }
hipError_t hipDeviceGetAttribute(int *v, hipDeviceAttribute_t, int) { *v = 256; return hipSuccess; }
hipError_t hipRuntimeGetVersion(int *v) { *v = 70200000; return hipSuccess; }
hipError_t hipGetLastError(void) { return hipSuccess; }
const char *hipGetErrorString(hipError_t) { return "stub runtime"; }
hipError_t hipMalloc(void **p, size_t n) { *p = std::malloc(n ? n : 1); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipFree(void *p) { std::free(p); return hipSuccess; }
hipError_t hipGetSymbolAddress(void **p, const void *) { static void *buf = std::calloc(1, 32u << 20); *p = buf; return hipSuccess; }
hipError_t hipDeviceSynchronize(void) { return hipSuccess; }
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t) { *ms = 0.25f; return hipSuccess; }
hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned)
{
    Ev *ev = new Ev();
    { std::lock_guard<std::mutex> g(g_all_mu); g_all[ev] = 1; }
    *e = reinterpret_cast<hipEvent_t>(ev);
    return hipSuccess;
}
hipError_t hipEventCreate(hipEvent_t *e) { return hipEventCreateWithFlags(e, 0); }
hipError_t hipEventDestroy(hipEvent_t e)
{
    Ev *ev = reinterpret_cast<Ev *>(e);
    { std::lock_guard<std::mutex> g(g_all_mu); g_all.erase(ev); }
    delete ev;
    return hipSuccess;
}
hipError_t hipEventRecord(hipEvent_t e, hipStream_t)
{
    reinterpret_cast<Ev *>(e)->records.fetch_add(1, std::memory_order_release);
    return hipSuccess;
}
hipError_t hipStreamWaitEvent(hipStream_t s, hipEvent_t e, unsigned)
{
    Ev *ev = reinterpret_cast<Ev *>(e);
    const long have = ev->records.load(std::memory_order_acquire);
    std::lock_guard<std::mutex> g(ev->mu);
    const long n = ev->waits[s]++ - ev->wait_base[s];
    if (g_phase == 2) {
        const long w = ev->per_round.count(s) ? ev->per_round[s] : 0;
        if (w > 0) {
            g_waits_checked++;
            if (have - ev->rec_base < n / w + 1) g_violations++;
        }
    }
    return hipSuccess;
}
hipError_t hipStreamBeginCapture(hipStream_t, hipStreamCaptureMode) { return hipErrorNotSupported; }
hipError_t hipStreamEndCapture(hipStream_t, hipGraph_t *g) { *g = nullptr; return hipErrorNotSupported; }
hipError_t hipGraphInstantiate(hipGraphExec_t *, hipGraph_t, hipGraphNode_t *, char *, size_t) { return hipErrorNotSupported; }
hipError_t hipGraphLaunch(hipGraphExec_t, hipStream_t) { return hipErrorNotSupported; }
hipError_t hipGraphDestroy(hipGraph_t) { return hipSuccess; }
hipError_t hipGraphExecDestroy(hipGraphExec_t) { return hipSuccess; }
}
