// Ceilings of one MI355X for the access shapes the library uses, measured with
// plain kernels that do none of the method's arithmetic: what HBM gives a
// read-only sweep, a fill, a 1-read-1-write copy and an 8-read-1-write kernel,
// and what the PCIe link gives copy kernels and the DMA engines, one way and
// both ways at once.  bench.py loads this file's shared library and prints the
// figures beside the nominal peaks (8 TB/s HBM3E, 64 GB/s per PCIe direction);
// built stand-alone (-DCEILINGS_MAIN) it is a program for rocprofv3.
//
// Not part of the product library and not used by it.
//
// HBM kernels: one wavefront per workgroup, one 16-byte vector per lane (a
// wavefront covers 1 KiB contiguously), non-temporal loads and stores, one
// workgroup per tile: the launch shape of the library's reduce and copy
// kernels.  Every launch touches at least 2 GiB that the previous launch did
// not touch (two buffer sets, used in turn), so nothing is served by the
// 256 MB memory-side cache.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr size_t kMiB = 1ull << 20;
constexpr size_t kSlice = 256 * kMiB;  // one simulated rank's message
constexpr int kStreams = 8;            // inputs of the many-stream kernels
constexpr size_t kBlock = kSlice * kStreams;  // 2 GiB: one buffer set

struct Fail {
    std::string what;
};

#define CK(expr)                                                                          \
    do {                                                                                  \
        hipError_t e_ = (expr);                                                           \
        if (e_ != hipSuccess) throw Fail{std::string(#expr) + ": " + hipGetErrorString(e_)}; \
    } while (0)

__device__ __forceinline__ u32x4 ldnt(const u32x4* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void stnt(u32x4* p, u32x4 v) { __builtin_nontemporal_store(v, p); }

// Read nvec vectors; the store is never taken for the data this program writes
// (every word is odd), it only keeps the loads alive.
__global__ void k_read(const u32x4* in, u32x4* sink, size_t nvec) {
    const size_t i = (size_t)blockIdx.x * 64 + threadIdx.x;
    if (i >= nvec) return;
    u32x4 v = ldnt(in + i);
    if ((v.x | v.y | v.z | v.w) == 0u) stnt(sink + (i & 63), v);
}

// Eight streams, one tile of each per wavefront, one load in flight at a time
// (the next load's index depends on the value just loaded).
template <bool STORE>
__global__ void k_xor8(const u32x4* in, u32x4* out, size_t nvec_per_stream) {
    size_t i = (size_t)blockIdx.x * 64 + threadIdx.x;
    if (i >= nvec_per_stream) return;
    const size_t stride = kSlice / 16;
    u32x4 acc = ldnt(in + i);
#pragma unroll
    for (int r = 1; r < kStreams; ++r) {
        asm volatile("" : "+v"(i) : "v"(acc.x));
        u32x4 v = ldnt(in + (size_t)r * stride + i);
        acc ^= v;
    }
    if (STORE)
        stnt(out + i, acc);
    else if ((acc.x | acc.y | acc.z | acc.w) == 0x80000000u)
        stnt(out + (i & 63), acc);
}

// The same with all eight loads issued before the first use.
__global__ void k_xor8_all(const u32x4* in, u32x4* out, size_t nvec_per_stream) {
    const size_t i = (size_t)blockIdx.x * 64 + threadIdx.x;
    if (i >= nvec_per_stream) return;
    const size_t stride = kSlice / 16;
    u32x4 v[kStreams];
#pragma unroll
    for (int r = 0; r < kStreams; ++r) v[r] = ldnt(in + (size_t)r * stride + i);
    u32x4 acc = v[0];
#pragma unroll
    for (int r = 1; r < kStreams; ++r) acc ^= v[r];
    stnt(out + i, acc);
}

template <int THREADS>
__global__ void k_fill(u32x4* out, size_t nvec, uint32_t word) {
    const size_t i = (size_t)blockIdx.x * THREADS + threadIdx.x;
    if (i < nvec) stnt(out + i, u32x4{word, word, word, word});
}

__global__ void k_copy(const u32x4* in, u32x4* out, size_t nvec) {
    const size_t i = (size_t)blockIdx.x * 64 + threadIdx.x;
    if (i < nvec) stnt(out + i, ldnt(in + i));
}

// PCIe: a fixed, small grid of 256-thread workgroups striding over the buffer,
// two vectors in flight per lane (the host path's copy shape).
__global__ void k_link_copy(const u32x4* in, u32x4* out, size_t nvec) {
    const size_t nthreads = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + nthreads < nvec; i += 2 * nthreads) {
        u32x4 a = in[i], b = in[i + nthreads];
        out[i] = a;
        out[i + nthreads] = b;
    }
    if (i < nvec) out[i] = in[i];
}

double median(std::vector<double> v) {
    std::sort(v.begin(), v.end());
    const size_t n = v.size();
    return (n & 1) ? v[n / 2] : 0.5 * (v[n / 2 - 1] + v[n / 2]);
}

struct Timer {
    hipEvent_t a, b;
    Timer() {
        CK(hipEventCreate(&a));
        CK(hipEventCreate(&b));
    }
    ~Timer() {
        (void)hipEventDestroy(a);
        (void)hipEventDestroy(b);
    }
};

// Median milliseconds of `reps` launches after `warm` untimed ones; launch(k)
// enqueues launch number k on stream 0.
template <class F>
double time_launches(int warm, int reps, F launch) {
    std::vector<Timer> t(reps);
    for (int k = 0; k < warm; ++k) launch(k);
    for (int k = 0; k < reps; ++k) {
        CK(hipEventRecord(t[k].a, 0));
        launch(warm + k);
        CK(hipEventRecord(t[k].b, 0));
    }
    CK(hipDeviceSynchronize());
    std::vector<double> ms;
    for (auto& e : t) {
        float x = 0;
        CK(hipEventElapsedTime(&x, e.a, e.b));
        ms.push_back(x);
    }
    return median(ms);
}

struct Json {
    std::string s = "{";
    bool first = true;
    void key(const char* k) {
        if (!first) s += ", ";
        first = false;
        s += "\"";
        s += k;
        s += "\": ";
    }
    void num(const char* k, double v) {
        char buf[64];
        snprintf(buf, sizeof buf, "%.6g", v);
        key(k);
        s += buf;
    }
    void str(const char* k, const char* v) {
        key(k);
        s += "\"";
        s += v;
        s += "\"";
    }
    void raw(const char* k, const std::string& v) {
        key(k);
        s += v;
    }
    std::string done() { return s + "}"; }
};

void hbm_ceilings(Json& out, int reps) {
    char* set[2] = {nullptr, nullptr};
    char* sink = nullptr;
    CK(hipMalloc((void**)&set[0], kBlock));
    CK(hipMalloc((void**)&set[1], kBlock));
    CK(hipMalloc((void**)&sink, 4096));
    try {
        const size_t nvec = kBlock / 16;
        const unsigned tiles = (unsigned)(nvec / 64);
        for (int s = 0; s < 2; ++s)
            hipLaunchKernelGGL(k_fill<256>, dim3((unsigned)(nvec / 256)), dim3(256), 0, 0, (u32x4*)set[s], nvec,
                               0x3f803f81u + 2u * s);
        CK(hipDeviceSynchronize());
        Json j;
        auto rate = [&](const char* name, double bytes, double ms) {
            j.num(name, bytes / ms / 1e6);  // GB/s
        };
        const int warm = 2;
        double ms;
        ms = time_launches(warm, reps, [&](int k) {
            hipLaunchKernelGGL(k_read, dim3(tiles), dim3(64), 0, 0, (const u32x4*)set[k & 1], (u32x4*)sink, nvec);
        });
        rate("read_one_stream_2GiB", (double)kBlock, ms);
        const size_t per = kSlice / 16;
        ms = time_launches(warm, reps, [&](int k) {
            hipLaunchKernelGGL(k_xor8<false>, dim3((unsigned)(per / 64)), dim3(64), 0, 0, (const u32x4*)set[k & 1],
                               (u32x4*)sink, per);
        });
        rate("read_eight_streams_2GiB", (double)kBlock, ms);
        ms = time_launches(warm, reps, [&](int k) {
            hipLaunchKernelGGL(k_fill<64>, dim3(tiles), dim3(64), 0, 0, (u32x4*)set[k & 1], nvec, 0x3f803f81u);
        });
        rate("fill_2GiB_one_wavefront_workgroups", (double)kBlock, ms);
        ms = time_launches(warm, reps, [&](int k) {
            hipLaunchKernelGGL(k_fill<256>, dim3((unsigned)(nvec / 256)), dim3(256), 0, 0, (u32x4*)set[k & 1], nvec,
                               0x3f803f81u);
        });
        rate("fill_2GiB_256_thread_workgroups", (double)kBlock, ms);
        // copy 1 GiB -> 1 GiB inside one set (2 GiB of traffic), sets in turn
        ms = time_launches(warm, reps, [&](int k) {
            hipLaunchKernelGGL(k_copy, dim3(tiles / 2), dim3(64), 0, 0, (const u32x4*)set[k & 1],
                               (u32x4*)(set[k & 1] + kBlock / 2), nvec / 2);
        });
        rate("copy_1GiB_to_1GiB", (double)kBlock, ms);
        // 8 reads + 1 write: inputs = one set, output = first slice of the other set
        ms = time_launches(warm, reps, [&](int k) {
            hipLaunchKernelGGL(k_xor8<true>, dim3((unsigned)(per / 64)), dim3(64), 0, 0, (const u32x4*)set[k & 1],
                               (u32x4*)set[(k + 1) & 1], per);
        });
        rate("xor_8_reads_1_write_one_load_in_flight", (double)(kBlock + kSlice), ms);
        // the same with 5632 bytes of (unused) LDS reserved per workgroup: a compute unit then holds 29
        // wavefronts instead of 32
        ms = time_launches(warm, reps, [&](int k) {
            hipLaunchKernelGGL(k_xor8<true>, dim3((unsigned)(per / 64)), dim3(64), 5632, 0, (const u32x4*)set[k & 1],
                               (u32x4*)set[(k + 1) & 1], per);
        });
        rate("xor_8_reads_1_write_one_load_in_flight_29_waves_per_cu", (double)(kBlock + kSlice), ms);
        ms = time_launches(warm, reps, [&](int k) {
            hipLaunchKernelGGL(k_xor8_all, dim3((unsigned)(per / 64)), dim3(64), 0, 0, (const u32x4*)set[k & 1],
                               (u32x4*)set[(k + 1) & 1], per);
        });
        rate("xor_8_reads_1_write_all_loads_in_flight", (double)(kBlock + kSlice), ms);
        j.str("unit", "GB/s");
        j.num("nominal_peak", 8000.0);
        j.str("shape", "64-thread workgroups, 16 B per lane, non-temporal, >= 2 GiB cold per launch, median");
        j.num("launches_timed", reps);
        out.raw("hbm", j.done());
    } catch (...) {
        (void)hipFree(set[0]);
        (void)hipFree(set[1]);
        (void)hipFree(sink);
        throw;
    }
    CK(hipFree(set[0]));
    CK(hipFree(set[1]));
    CK(hipFree(sink));
}

// One PCIe leg: `reps` transfers of `bytes` back to back on `stream`.
struct Leg {
    bool up;       // device -> pinned host memory
    bool kernel;   // copy kernel (else hipMemcpyAsync on a DMA engine)
    unsigned blocks;
};

void enqueue_leg(const Leg& leg, char* dev, char* host, size_t bytes, int reps, hipStream_t stream) {
    for (int k = 0; k < reps; ++k) {
        const char* src = leg.up ? dev : host;
        char* dst = leg.up ? host : dev;
        if (leg.kernel)
            hipLaunchKernelGGL(k_link_copy, dim3(leg.blocks), dim3(256), 0, stream, (const u32x4*)src, (u32x4*)dst,
                               bytes / 16);
        else
            CK(hipMemcpyAsync(dst, src, bytes, leg.up ? hipMemcpyDeviceToHost : hipMemcpyHostToDevice, stream));
    }
}

void pcie_ceilings(Json& out, int reps) {
    const size_t bytes = 28 * kMiB;  // one pipeline step of the host path: 7 peers x 4 MiB
    char *dev[2] = {nullptr, nullptr}, *host[2] = {nullptr, nullptr};
    hipStream_t st[2] = {nullptr, nullptr};
    for (int i = 0; i < 2; ++i) {
        CK(hipMalloc((void**)&dev[i], bytes));
        CK(hipHostMalloc((void**)&host[i], bytes, hipHostMallocDefault));
        memset(host[i], 0x5a, bytes);
        CK(hipMemset(dev[i], 0x3c, bytes));
        CK(hipStreamCreateWithFlags(&st[i], hipStreamNonBlocking));
    }
    CK(hipDeviceSynchronize());
    Json j;
    auto run = [&](const char* name, const Leg* a, const Leg* b) {
        // untimed pass, then a timed one: wall clock around both streams
        for (int pass = 0; pass < 2; ++pass) {
            Timer ta, tb;
            CK(hipDeviceSynchronize());
            const auto t0 = std::chrono::steady_clock::now();
            if (a) {
                CK(hipEventRecord(ta.a, st[0]));
                enqueue_leg(*a, dev[0], host[0], bytes, reps, st[0]);
                CK(hipEventRecord(ta.b, st[0]));
            }
            if (b) {
                CK(hipEventRecord(tb.a, st[1]));
                enqueue_leg(*b, dev[1], host[1], bytes, reps, st[1]);
                CK(hipEventRecord(tb.b, st[1]));
            }
            CK(hipDeviceSynchronize());
            const double wall_ms =
                std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
            if (pass == 0) continue;
            Json r;
            float ms = 0;
            if (a) {
                CK(hipEventElapsedTime(&ms, ta.a, ta.b));
                r.num(a->up ? "device_to_host" : "host_to_device", (double)bytes * reps / ms / 1e6);
            }
            if (b) {
                CK(hipEventElapsedTime(&ms, tb.a, tb.b));
                r.num(b->up ? "device_to_host" : "host_to_device", (double)bytes * reps / ms / 1e6);
            }
            r.num("wall_ms", wall_ms);
            j.raw(name, r.done());
        }
    };
    const Leg up_dma{true, false, 0}, down_dma{false, false, 0};
    run("dma_one_way_up", &up_dma, nullptr);
    run("dma_one_way_down", nullptr, &down_dma);
    run("dma_both_ways", &up_dma, &down_dma);
    for (unsigned blocks : {16u, 64u, 256u}) {
        const Leg up_k{true, true, blocks}, down_k{false, true, blocks};
        char name[64];
        snprintf(name, sizeof name, "kernel_%u_workgroups_one_way_up", blocks);
        run(name, &up_k, nullptr);
        snprintf(name, sizeof name, "kernel_%u_workgroups_one_way_down", blocks);
        run(name, nullptr, &down_k);
        snprintf(name, sizeof name, "kernel_%u_workgroups_both_ways", blocks);
        run(name, &up_k, &down_k);
        snprintf(name, sizeof name, "kernel_%u_workgroups_up_dma_down", blocks);
        run(name, &up_k, &down_dma);
    }
    j.str("unit", "GB/s per direction");
    j.num("nominal_peak", 64.0);
    j.num("transfer_MiB", (double)bytes / kMiB);
    j.num("transfers_per_leg", reps);
    out.raw("pcie", j.done());
    for (int i = 0; i < 2; ++i) {
        CK(hipStreamDestroy(st[i]));
        CK(hipFree(dev[i]));
        CK(hipHostFree(host[i]));
    }
}

}  // namespace

// Runs the probes on the current device and writes one JSON object (NUL
// terminated) to json_out.  what: bit 0 = HBM, bit 1 = PCIe.  Returns 0, or 1
// with an error message in json_out.
extern "C" int flex_ceilings_run(char* json_out, size_t cap, int what, int reps) {
    if (!json_out || cap == 0) return 1;
    if (reps < 1) reps = 6;
    try {
        Json out;
        if (what & 1) hbm_ceilings(out, reps);
        if (what & 2) pcie_ceilings(out, reps * 2);
        snprintf(json_out, cap, "%s", out.done().c_str());
        return 0;
    } catch (const Fail& f) {
        snprintf(json_out, cap, "%s", f.what.c_str());
        return 1;
    }
}

#ifdef CEILINGS_MAIN
int main(int argc, char** argv) {
    int what = 3, reps = 6;
    for (int i = 1; i < argc; ++i) {
        if (!strcmp(argv[i], "--hbm")) what = 1;
        else if (!strcmp(argv[i], "--pcie")) what = 2;
        else if (!strcmp(argv[i], "--reps") && i + 1 < argc) reps = atoi(argv[++i]);
    }
    static char buf[1 << 16];
    const int rc = flex_ceilings_run(buf, sizeof buf, what, reps);
    puts(buf);
    return rc;
}
#endif
