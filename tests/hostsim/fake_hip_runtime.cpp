// A stand-in for the HIP runtime that runs on the CPU, for sanitizer builds of the library's host code.
//
// The host side of libdft3d (plan creation, matrix generation and upload, argument checks, the
// sequencing of passes, every launch-parameter computation in front of a kernel) is compiled host-only
// with AddressSanitizer and UndefinedBehaviorSanitizer and linked against this file instead of
// libamdhip64.  "Device" memory is host memory with a registry of live allocations, so ASan sees every
// upload; a kernel launch executes nothing but is recorded -- kernel name, grid, block, dynamic LDS --
// and, for the kernels whose first argument describes their tensors, checked: the region the launch
// reads and the region it writes must lie inside live allocations.  TEST INFRASTRUCTURE ONLY.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include <cxxabi.h>
#include <sys/mman.h>

#include "dft3d_internal.h"
#include "hostsim.h"

namespace {

struct Alloc {
    size_t bytes;
};
// The registries are built on first use: the code objects register their kernels from static
// initialisers that may run before this file's own.
struct State {
    std::map<uintptr_t, Alloc> allocs;                // base -> size
    std::map<const void*, std::string> kernels;       // host stub address -> demangled name
    std::map<const void*, size_t> max_dynamic_lds;    // set by hipFuncSetAttribute
    std::map<const void*, void*> symbols;             // host shadow of a __device__ variable -> its "device" copy
    std::vector<hostsim_launch> log;
    std::string failure;
};
State& state()
{
    static State* s = new State();                    // (never destroyed: used until the process ends)
    return *s;
}
#define g_allocs (state().allocs)
#define g_kernels (state().kernels)
#define g_max_dynamic_lds (state().max_dynamic_lds)
#define g_symbols (state().symbols)
#define g_log (state().log)
#define g_failure (state().failure)
hipError_t g_last_error = hipSuccess;

struct CallConfig {
    dim3 grid, block;
    size_t shmem;
    hipStream_t stream;
};
thread_local std::vector<CallConfig> t_configs;

void fail(const std::string& what)
{
    if (g_failure.empty()) g_failure = what;
}

// the live allocation that holds [p, p + bytes), or nullptr
const std::pair<const uintptr_t, Alloc>* find_alloc(const void* p, size_t bytes)
{
    const uintptr_t a = (uintptr_t)p;
    auto it = g_allocs.upper_bound(a);
    if (it == g_allocs.begin()) return nullptr;
    --it;
    if (a < it->first || a + bytes > it->first + it->second.bytes) return nullptr;
    return &*it;
}

std::string demangle(const char* name)
{
    int status = 0;
    char* d = abi::__cxa_demangle(name, nullptr, nullptr, &status);
    std::string s = (status == 0 && d) ? d : name;
    free(d);
    return s;
}

// the integer template arguments of "k_name<16, 32, 2>(...)"
std::vector<long> template_ints(const std::string& name)
{
    std::vector<long> v;
    const size_t a = name.find('<');
    const size_t b = name.find(">(");
    if (a == std::string::npos || b == std::string::npos || b < a) return v;
    const std::string inner = name.substr(a + 1, b - a - 1);
    size_t pos = 0;
    while (pos < inner.size()) {
        size_t end = inner.find(',', pos);
        if (end == std::string::npos) end = inner.size();
        const std::string tok = inner.substr(pos, end - pos);
        char* e = nullptr;
        const long val = strtol(tok.c_str(), &e, 10);
        v.push_back((e && e != tok.c_str()) ? val : (tok.find("true") != std::string::npos ? 1 : 0));
        pos = end + 1;
    }
    return v;
}

void check_region(const std::string& kernel, const char* what, const void* p, int64_t bytes)
{
    if (bytes <= 0) return;
    if (!p || !find_alloc(p, (size_t)bytes)) {
        char buf[512];
        snprintf(buf, sizeof(buf), "%s: the %s region [%p, +%lld bytes) is not inside a live allocation", kernel.c_str(),
                 what, p, (long long)bytes);
        fail(buf);
    }
}

}  // namespace

// ---- what the test driver sees --------------------------------------------------------------------
extern "C" {

size_t hostsim_launch_count(void) { return g_log.size(); }
const hostsim_launch* hostsim_launches(void) { return g_log.data(); }
void hostsim_clear_log(void) { g_log.clear(); }
void* hostsim_reserve(size_t bytes)
{
    void* p = mmap(nullptr, bytes ? bytes : 1, PROT_NONE, MAP_PRIVATE | MAP_ANONYMOUS | MAP_NORESERVE, -1, 0);
    if (p == MAP_FAILED) return nullptr;
    g_allocs[(uintptr_t)p] = Alloc{bytes};
    return p;
}
void hostsim_release(void* p, size_t bytes)
{
    g_allocs.erase((uintptr_t)p);
    munmap(p, bytes ? bytes : 1);
}
const char* hostsim_failure(void) { return g_failure.empty() ? nullptr : g_failure.c_str(); }
size_t hostsim_live_allocations(void) { return g_allocs.size(); }

// ---- code-object registration (called from static initialisers of the host-only objects) -----------
void** __hipRegisterFatBinary(const void*)
{
    static void* dummy = nullptr;
    return &dummy;
}
void __hipUnregisterFatBinary(void**) {}
void __hipRegisterFunction(void**, const void* hostFunction, char*, const char* deviceName, unsigned, void*, void*, void*,
                           void*, int*)
{
    g_kernels[hostFunction] = demangle(deviceName);
}
void __hipRegisterVar(void**, void* var, char*, char*, int, size_t size, int, int)
{
    void* dev = calloc(1, size ? size : 1);
    g_symbols[var] = dev;
    g_allocs[(uintptr_t)dev] = Alloc{size};
}

hipError_t __hipPushCallConfiguration(dim3 grid, dim3 block, size_t shmem, hipStream_t stream)
{
    t_configs.push_back(CallConfig{grid, block, shmem, stream});
    return hipSuccess;
}
hipError_t __hipPopCallConfiguration(dim3* grid, dim3* block, size_t* shmem, hipStream_t* stream)
{
    if (t_configs.empty()) return hipErrorInvalidValue;
    const CallConfig c = t_configs.back();
    t_configs.pop_back();
    *grid = c.grid;
    *block = c.block;
    *shmem = c.shmem;
    *stream = c.stream;
    return hipSuccess;
}

}  // extern "C"

// ---- runtime calls ---------------------------------------------------------------------------------
hipError_t hipMalloc(void** p, size_t bytes)
{
    if (!p) return hipErrorInvalidValue;
    if (bytes > ((size_t)1 << 40)) {          // what no GPU could give either
        *p = nullptr;
        return g_last_error = hipErrorOutOfMemory;
    }
    void* m = malloc(bytes ? bytes : 1);
    if (!m) return g_last_error = hipErrorOutOfMemory;
    g_allocs[(uintptr_t)m] = Alloc{bytes};
    *p = m;
    return hipSuccess;
}
hipError_t hipFree(void* p)
{
    if (!p) return hipSuccess;
    auto it = g_allocs.find((uintptr_t)p);
    if (it == g_allocs.end()) {
        fail("hipFree of a pointer that is not a live allocation");
        return hipErrorInvalidValue;
    }
    g_allocs.erase(it);
    free(p);
    return hipSuccess;
}
hipError_t hipMemcpy(void* dst, const void* src, size_t bytes, hipMemcpyKind kind)
{
    if (kind == hipMemcpyHostToDevice) check_region("hipMemcpy", "destination", dst, (int64_t)bytes);
    if (kind == hipMemcpyDeviceToHost) check_region("hipMemcpy", "source", src, (int64_t)bytes);
    memcpy(dst, src, bytes);
    return hipSuccess;
}
hipError_t hipGetLastError(void)
{
    const hipError_t e = g_last_error;
    g_last_error = hipSuccess;
    return e;
}
const char* hipGetErrorString(hipError_t e) { return e == hipSuccess ? "no error" : "simulated HIP error"; }
hipError_t hipGetDevice(int* dev)
{
    *dev = 0;
    return hipSuccess;
}
hipError_t hipGetSymbolAddress(void** devPtr, const void* symbol)
{
    auto it = g_symbols.find(symbol);
    if (it == g_symbols.end()) return hipErrorInvalidSymbol;
    *devPtr = it->second;
    return hipSuccess;
}
hipError_t hipFuncSetAttribute(const void* func, hipFuncAttribute attr, int value)
{
    if (!g_kernels.count(func)) {
        fail("hipFuncSetAttribute on something that is not a registered kernel");
        return hipErrorInvalidDeviceFunction;
    }
    if (attr == hipFuncAttributeMaxDynamicSharedMemorySize) {
        if (value < 0 || value > 160 * 1024) {
            fail(g_kernels[func] + ": asks for more dynamic LDS than a CU has");
            return hipErrorInvalidValue;
        }
        g_max_dynamic_lds[func] = (size_t)value;
    }
    return hipSuccess;
}
hipError_t hipEventCreate(hipEvent_t* ev)
{
    *ev = (hipEvent_t)malloc(8);
    return hipSuccess;
}
hipError_t hipEventDestroy(hipEvent_t ev)
{
    free(ev);
    return hipSuccess;
}
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t)
{
    *ms = 0.0f;
    return hipSuccess;
}

hipError_t hipLaunchKernel(const void* func, dim3 grid, dim3 block, void** args, size_t shmem, hipStream_t)
{
    auto it = g_kernels.find(func);
    if (it == g_kernels.end()) {
        fail("launch of a function that is not a registered kernel");
        return g_last_error = hipErrorInvalidDeviceFunction;
    }
    const std::string& name = it->second;
    // launch limits of the hardware / runtime
    const uint64_t threads = (uint64_t)block.x * block.y * block.z;
    if (threads == 0 || threads > 1024 || grid.x == 0 || grid.y == 0 || grid.z == 0 || grid.y > 65535 || grid.z > 65535 ||
        (uint64_t)grid.x * block.x > 0xffffffffull)
        fail(name + ": launch shape outside the limits");
    const size_t lds_allowed = g_max_dynamic_lds.count(func) ? g_max_dynamic_lds[func] : 64 * 1024;
    if (shmem > lds_allowed) fail(name + ": more dynamic LDS than the kernel was configured for");

    hostsim_launch L{};
    L.name = name.c_str();          // (map nodes do not move)
    L.grid[0] = grid.x, L.grid[1] = grid.y, L.grid[2] = grid.z;
    L.block[0] = block.x, L.block[1] = block.y, L.block[2] = block.z;
    L.dynamic_lds = shmem;

    using namespace dft3d;
    auto starts = [&](const char* p) { return name.find(p) != std::string::npos; };
    if (starts("k_contract_f64<")) {
        const ContractArgs64& a = *(const ContractArgs64*)args[0];
        const int64_t hi = (a.O - 1) / a.Olo, lo = (a.O - 1 < a.Olo - 1) ? a.O - 1 : a.Olo - 1;
        L.src = a.X, L.dst = a.Y;
        L.src_bytes = a.O * a.N * a.I * 16;
        L.dst_bytes = (hi * a.sYohi + lo * a.sYolo + (int64_t)(a.K - 1) * a.sYk + a.I) * 16;
        check_region(name, "matrix", a.M, (int64_t)2 * a.ld * a.rows * 8);
    } else if (starts("k_contract_s<") || starts("k_contract_c<") || starts("k_contract_sr<") ||
               starts("k_contract_bf16x3<")) {
        const ContractArgs& a = *(const ContractArgs*)args[0];
        const int64_t hi = (a.O - 1) / a.Olo, lo = (a.O - 1 < a.Olo - 1) ? a.O - 1 : a.Olo - 1;
        L.src = a.X, L.dst = a.Y;
        L.src_bytes = a.O * a.M.N * a.I * 8;
        L.dst_bytes = (hi * a.sYohi + lo * a.sYolo + (int64_t)(a.M.K - 1) * a.sYk + a.I) * 8;
        check_region(name, "matrix", a.M.re, (int64_t)2 * a.M.ld * a.M.rows * 4);
        if (starts("k_contract_bf16x3<"))
            check_region(name, "bf16 matrix planes", a.M.split, (int64_t)a.M.split_planes * a.M.split_ld * a.M.split_rows * 2);
    } else if (starts("k_fft_sr<")) {
        const FftStridedArgs& a = *(const FftStridedArgs*)args[0];
        const std::vector<long> t = template_ints(name);
        const int64_t N = t.size() >= 2 ? t[0] * t[1] : 0;
        L.src = a.X, L.dst = a.Y;
        L.src_bytes = ((a.O - 1) * a.inO + (N - 1) * a.inN + (a.Yn - 1) * a.inY + 16 * a.Zt) * 8;
        L.dst_bytes = ((a.O - 1) * a.outO + (N - 1) * a.outN + (a.Yn - 1) * a.outY + 16 * a.Zt) * 8;
        if (N <= 0) fail(name + ": cannot read the split from the kernel name");
    } else if (starts("k_fft_sn<")) {
        // (16*NAB) x (C*16) on a strided axis
        const FftStridedArgs& a = *(const FftStridedArgs*)args[0];
        const std::vector<long> t = template_ints(name);
        const int64_t N = t.size() >= 2 ? 256 * t[0] * t[1] : 0;
        L.src = a.X, L.dst = a.Y;
        L.src_bytes = ((a.O - 1) * a.inO + (N - 1) * a.inN + (a.Yn - 1) * a.inY + 16 * a.Zt) * 8;
        L.dst_bytes = ((a.O - 1) * a.outO + (N - 1) * a.outN + (a.Yn - 1) * a.outY + 16 * a.Zt) * 8;
        if (N <= 0) fail(name + ": cannot read the split from the kernel name");
        if (t.size() >= 2 && 3 * 16 * t[1] * a.inN + 16 > 0xffffffffll) fail(name + ": 32-bit lane offsets of the loads overflow");
    } else if (starts("k_fft_zn<")) {
        const std::vector<long> t = template_ints(name);
        const int64_t N = t.size() >= 2 ? 256 * t[0] * t[1] : 0;
        const int64_t nrows = *(const int64_t*)args[2];
        L.src = *(const void* const*)args[0], L.dst = *(void* const*)args[1];
        L.src_bytes = L.dst_bytes = nrows * N * 8;
        if (N <= 0) fail(name + ": cannot read the split from the kernel name");
    } else if (starts("k_fft_zr<") || starts("k_fft_z<")) {
        const std::vector<long> t = template_ints(name);
        const int64_t N = t.size() >= 2 ? t[0] * t[1] : 0;
        const int64_t nrows = *(const int64_t*)args[2];
        L.src = *(const void* const*)args[0], L.dst = *(void* const*)args[1];
        L.src_bytes = L.dst_bytes = nrows * N * 8;
    } else if (starts("k_radix_tw<")) {
        // element-wise first stage on [O][R][I]: args in, out, pairs (= O * I / 2), I / 2, ..
        const std::vector<long> t = template_ints(name);
        const int64_t R = t.size() >= 1 ? t[0] : 0;
        const int64_t npairs = *(const int64_t*)args[2];
        L.src = *(const void* const*)args[0], L.dst = *(void* const*)args[1];
        L.src_bytes = L.dst_bytes = npairs * 2 * R * 8;
        if (R != 2 && R != 4 && R != 8) fail(name + ": cannot read the radix from the kernel name");
        if ((uint64_t)grid.x * 256 < (uint64_t)npairs) fail(name + ": grid does not cover the tensor");
    } else if (starts("k_kdft_small")) {
        const DeviceMatrix& Mx = *(const DeviceMatrix*)args[2];
        const DeviceMatrix& My = *(const DeviceMatrix*)args[3];
        const DeviceMatrix& Mz = *(const DeviceMatrix*)args[4];
        L.src = *(const void* const*)args[0], L.dst = *(void* const*)args[1];
        L.src_bytes = (int64_t)Mx.N * My.N * Mz.N * 8;
        L.dst_bytes = (int64_t)Mx.K * My.K * Mz.K * 8;
    }
    if (L.src) check_region(name, "input", L.src, L.src_bytes);
    if (L.dst) check_region(name, "output", L.dst, L.dst_bytes);
    g_log.push_back(L);
    return hipSuccess;
}
