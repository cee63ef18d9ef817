// A stand-in for the HIP runtime, for CPU-only tests of the library's host code: the request
// life cycle of iso_api.hip / iso_bind.hpp (device tables, graphs, the static scratch array) runs
// against it under AddressSanitizer and LeakSanitizer with no GPU.  "Device" memory is host heap,
// kernels are never run, and every object the library creates is counted, so that a run can end
// with the statement that nothing the library made is still alive.
#include <hip/hip_runtime_api.h>      // host API declarations only: this file is plain C++

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>

namespace {
std::mutex g_mu;
std::map<uintptr_t, size_t> g_allocs;          // live hipMalloc ranges
long g_graphs = 0, g_execs = 0, g_launches = 0, g_graph_launches = 0, g_nodes = 0;
alignas(256) unsigned char g_symbol_memory[64u << 20];      // what hipGetSymbolAddress hands out
struct StubGraph { int nodes; };
struct StubExec { int nodes; };
}  // namespace

extern "C" {
// what the compiler's kernel stubs and module constructor call
extern const char __hip_fatbin[8];
const char __hip_fatbin[8] = {0};
void **__hipRegisterFatBinary(const void *) { static void *h; return &h; }
void __hipRegisterFunction(void **, const void *, char *, const char *, unsigned, void *, void *, void *, void *, int *) {}
void __hipRegisterVar(void **, void *, char *, const char *, int, size_t, int, int) {}
void __hipUnregisterFatBinary(void **) {}
struct StubCall { dim3 grid, block; size_t shmem; hipStream_t stream; };
static thread_local StubCall g_call;
hipError_t __hipPushCallConfiguration(dim3 grid, dim3 block, size_t shmem, hipStream_t stream) {
    g_call = StubCall{grid, block, shmem, stream};
    return hipSuccess;
}
hipError_t __hipPopCallConfiguration(dim3 *grid, dim3 *block, size_t *shmem, hipStream_t *stream) {
    *grid = g_call.grid; *block = g_call.block; *shmem = g_call.shmem; *stream = g_call.stream;
    return hipSuccess;
}

hipError_t hipGetLastError(void) { return hipSuccess; }
hipError_t hipGetDevice(int *dev) { *dev = 0; return hipSuccess; }
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }

hipError_t hipMalloc(void **ptr, size_t bytes) {
    void *q = std::malloc(bytes ? bytes : 1);
    if (!q) return hipErrorOutOfMemory;
    std::lock_guard<std::mutex> lock(g_mu);
    g_allocs[(uintptr_t)q] = bytes;
    *ptr = q;
    return hipSuccess;
}
hipError_t hipFree(void *ptr) {
    if (!ptr) return hipSuccess;
    std::lock_guard<std::mutex> lock(g_mu);
    auto it = g_allocs.find((uintptr_t)ptr);
    if (it == g_allocs.end()) return hipErrorInvalidValue;
    g_allocs.erase(it);
    std::free(ptr);
    return hipSuccess;
}
hipError_t hipMemcpy(void *dst, const void *src, size_t bytes, hipMemcpyKind) {
    std::memcpy(dst, src, bytes);
    return hipSuccess;
}
hipError_t hipMemGetAddressRange(hipDeviceptr_t *base, size_t *size, hipDeviceptr_t ptr) {
    std::lock_guard<std::mutex> lock(g_mu);
    auto it = g_allocs.upper_bound((uintptr_t)ptr);
    if (it == g_allocs.begin()) return hipErrorInvalidValue;
    --it;
    if ((uintptr_t)ptr >= it->first + (it->second ? it->second : 1)) return hipErrorInvalidValue;
    *base = (hipDeviceptr_t)it->first;
    *size = it->second;
    return hipSuccess;
}
hipError_t hipGetSymbolAddress(void **ptr, const void *) { *ptr = g_symbol_memory; return hipSuccess; }
hipError_t hipLaunchKernel(const void *, dim3, dim3, void **, size_t, hipStream_t) { ++g_launches; return hipSuccess; }

hipError_t hipGraphCreate(hipGraph_t *g, unsigned) { *g = (hipGraph_t) new StubGraph{0}; ++g_graphs; return hipSuccess; }
hipError_t hipGraphAddKernelNode(hipGraphNode_t *node, hipGraph_t g, const hipGraphNode_t *, size_t,
                                 const hipKernelNodeParams *p) {
    if (!p || !p->func || !p->kernelParams || !p->kernelParams[0]) return hipErrorInvalidValue;
    StubGraph *sg = (StubGraph *)g;
    *node = (hipGraphNode_t)(uintptr_t)(++sg->nodes);
    ++g_nodes;
    return hipSuccess;
}
hipError_t hipGraphInstantiate(hipGraphExec_t *e, hipGraph_t g, hipGraphNode_t *, char *, size_t) {
    *e = (hipGraphExec_t) new StubExec{((StubGraph *)g)->nodes};
    ++g_execs;
    return hipSuccess;
}
hipError_t hipGraphLaunch(hipGraphExec_t e, hipStream_t) {
    if (!e) return hipErrorInvalidValue;
    ++g_graph_launches;
    return hipSuccess;
}
hipError_t hipGraphDestroy(hipGraph_t g) { delete (StubGraph *)g; --g_graphs; return hipSuccess; }
hipError_t hipGraphExecDestroy(hipGraphExec_t e) { delete (StubExec *)e; --g_execs; return hipSuccess; }

// ---- for the test driver ----
void *stub_device_alloc(size_t bytes) { void *q = nullptr; return hipMalloc(&q, bytes) == hipSuccess ? q : nullptr; }
void stub_device_free(void *q) { (void)hipFree(q); }
long stub_live_allocations(void) { std::lock_guard<std::mutex> lock(g_mu); return (long)g_allocs.size(); }
long stub_live_graph_objects(void) { return g_graphs + g_execs; }
long stub_kernel_launches(void) { return g_launches; }
long stub_graph_launches(void) { return g_graph_launches; }
long stub_graph_nodes(void) { return g_nodes; }
}

// Planted mistake for the test of the test: a build of the library in which hipFree is renamed to
// this (-DhipFree=stub_forgetful_free) never releases its device tables.
extern "C" hipError_t stub_forgetful_free(void *) { return hipSuccess; }
