// Optional per-kernel timing: while enabled, every kernel launch of the library is bracketed by two HIP
// events recorded on the caller's stream.  Reading a slot waits for its events and accumulates elapsed time,
// launch count and the algorithmic operations and bytes of those launches.  Host-side bookkeeping only.
#include <mutex>
#include <string>
#include <vector>

#include "mq_common.h"

namespace mq {

namespace {
struct Pair {
    hipEvent_t a, b;
};
struct Slot {
    std::string name;
    long long launches = 0;
    double ms = 0, ops = 0, bytes = 0;
    std::vector<Pair> pending;
};
std::mutex g_mu;
bool g_on = false;
int g_filter_slot = -1;   // -1: every kernel; else only launches of this slot ...
int g_filter_stride = 1;  // ... and of those only every stride-th
long g_filter_count = 0;
std::vector<Slot> g_slots;
std::vector<Pair> g_free;

void init_slots() {
    if (!g_slots.empty()) return;
    g_slots.resize(prof_num_slots());
    g_slots[PROF_ACT_MINMAX].name = "mq::act_minmax_kernel";
    g_slots[PROF_ACT_QUANTIZE].name = "mq::act_quantize_kernel";
    g_slots[PROF_BOS_ROWS].name = "mq::bos_rows_kernel<8>";
}
}  // namespace

int prof_num_slots() { return PROF_BOS_ROWS + 1; }

// What an event pair adds to the kernel it brackets (dispatch latency on either side): measured once, on the
// stream given, with a single-workgroup kernel that spins for a known 20 us of the constant 100 MHz clock.
__global__ void prof_spin_kernel(long long ticks) {
    const long long t0 = wall_clock64();
    while (wall_clock64() - t0 < ticks) {
    }
}

// Plain copy of a known size: the reference that HBM traffic counters are scaled by.
__global__ __launch_bounds__(256) void prof_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, long n16) {
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (long)gridDim.x * blockDim.x) dst[i] = src[i];
}

int prof_copy(void* dst, const void* src, size_t bytes, hipStream_t st) {
    if (!dst || !src || bytes % 16 != 0 || ((uintptr_t)dst | (uintptr_t)src) % 16 != 0) return MQ_ERR_BAD_ARG;
    hipLaunchKernelGGL(prof_copy_kernel, dim3(4096), dim3(256), 0, st, (const uint4*)src, (uint4*)dst, (long)(bytes / 16));
    MQ_HIP_CHECK_LAUNCH();
    return MQ_OK;
}

static double g_overhead_us = -1.0;

double prof_bracket_overhead_us(hipStream_t st) {
    if (g_overhead_us >= 0.0) return g_overhead_us;
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return 0.0;
    double best = 1e30;
    for (int i = 0; i < 12; ++i) {
        (void)hipEventRecord(a, st);
        hipLaunchKernelGGL(prof_spin_kernel, dim3(1), dim3(64), 0, st, 2000LL);
        (void)hipEventRecord(b, st);
        if (hipEventSynchronize(b) != hipSuccess) break;
        float ms = 0;
        if (hipEventElapsedTime(&ms, a, b) == hipSuccess && i >= 2 && ms * 1e3 < best) best = ms * 1e3;
    }
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    g_overhead_us = best < 1e29 ? (best > 20.0 ? best - 20.0 : 0.0) : 0.0;
    return g_overhead_us;
}

int prof_gemm_slot(int family, int bits, int tile) {
    const int b = bits == 2 ? 0 : bits == 3 ? 1 : bits == 4 ? 2 : bits == 8 ? 3 : 4;
    return (family * PROF_GEMM_BITS + b) * PROF_GEMM_TILES + tile;
}

bool prof_enabled() { return g_on; }

bool prof_wants(int slot) {
    if (g_filter_slot < 0) return true;
    if (slot != g_filter_slot) return false;
    std::lock_guard<std::mutex> lk(g_mu);
    return (g_filter_count++ % g_filter_stride) == 0;
}

int prof_filter(int slot, int stride) {
    std::lock_guard<std::mutex> lk(g_mu);
    init_slots();
    if (slot >= (int)g_slots.size() || stride < 1) return MQ_ERR_BAD_ARG;
    g_filter_slot = slot;
    g_filter_stride = stride;
    g_filter_count = 0;
    return MQ_OK;
}

void prof_name_slot(int slot, const char* name) {
    std::lock_guard<std::mutex> lk(g_mu);
    init_slots();
    g_slots[slot].name = name;
}

int prof_enable(int on) {
    std::lock_guard<std::mutex> lk(g_mu);
    init_slots();
    g_on = on != 0;
    return MQ_OK;
}

bool prof_begin(hipStream_t st, hipEvent_t* a, hipEvent_t* b) {
    std::lock_guard<std::mutex> lk(g_mu);
    Pair p;
    if (!g_free.empty()) {
        p = g_free.back();
        g_free.pop_back();
    } else {
        if (hipEventCreate(&p.a) != hipSuccess) return false;
        if (hipEventCreate(&p.b) != hipSuccess) {
            (void)hipEventDestroy(p.a);
            return false;
        }
    }
    if (hipEventRecord(p.a, st) != hipSuccess) {
        g_free.push_back(p);
        return false;
    }
    *a = p.a;
    *b = p.b;
    return true;
}

void prof_end(hipEvent_t a, hipEvent_t b, hipStream_t st, int slot, double ops, double bytes) {
    std::lock_guard<std::mutex> lk(g_mu);
    (void)hipEventRecord(b, st);
    Slot& s = g_slots[slot];
    s.pending.push_back(Pair{a, b});
    s.launches += 1;
    s.ops += ops;
    s.bytes += bytes;
}

int prof_read(int slot, char* name, int name_cap, long long* launches, double* ms, double* ops, double* bytes) {
    std::lock_guard<std::mutex> lk(g_mu);
    init_slots();
    if (slot < 0 || slot >= (int)g_slots.size()) return MQ_ERR_BAD_ARG;
    Slot& s = g_slots[slot];
    for (Pair& p : s.pending) {
        float t = 0;
        if (hipEventSynchronize(p.b) != hipSuccess || hipEventElapsedTime(&t, p.a, p.b) != hipSuccess) {
            set_hip_error((int)hipGetLastError());
            return MQ_ERR_HIP;
        }
        s.ms += t;
        g_free.push_back(p);
    }
    s.pending.clear();
    if (name && name_cap > 0) {
        snprintf(name, name_cap, "%s", s.name.c_str());
    }
    if (launches) *launches = s.launches;
    if (ms) *ms = s.ms;
    if (ops) *ops = s.ops;
    if (bytes) *bytes = s.bytes;
    return MQ_OK;
}

int prof_reset() {
    std::lock_guard<std::mutex> lk(g_mu);
    init_slots();
    for (Slot& s : g_slots) {
        for (Pair& p : s.pending) {
            (void)hipEventSynchronize(p.b);
            g_free.push_back(p);
        }
        s.pending.clear();
        s.launches = 0;
        s.ms = s.ops = s.bytes = 0;
    }
    return MQ_OK;
}

}  // namespace mq
