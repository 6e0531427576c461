// flex_allreduce_staged_noalloc: the split AllReduce for callers that cannot
// allocate.  The staged part of the message goes through a file-scope device
// array instead of buffers a communicator allocated, everything runs on the
// caller's stream, and the call makes no allocation of any kind.
#include <hip/hip_runtime.h>

#include <mutex>

#include "flexlink_internal.h"

namespace {

// Transit buffer for the staged part: all peers' pieces back to back.  32 MiB
// holds one pipeline step of the host path's default size (7 peers x 4 MiB).
// Every GPU the library runs on holds its own copy until the process ends.
constexpr size_t kScratchBytes = 32u << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mutex;
unsigned char* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, once looked up
int g_num_cus[kMaxDevices];

// The address of this device's copy of `scratch` (looked up once per device,
// with that device current).  The array's name itself is only a host-side
// stand-in and is never handed to a kernel or a copy.
int scratch_for_current_device(unsigned char** ptr, int* cus) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return flex::fail(FLEX_ERR_HIP, "flex_allreduce_staged_noalloc: hipGetDevice failed: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices)
        return flex::fail(FLEX_ERR_UNSUPPORTED, "flex_allreduce_staged_noalloc: device index %d not supported", dev);
    std::lock_guard<std::mutex> lock(g_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return flex::fail(FLEX_ERR_HIP, "flex_allreduce_staged_noalloc: hipGetSymbolAddress failed: %s",
                              hipGetErrorString(e));
        int n = 0;
        e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess || n <= 0)
            return flex::fail(FLEX_ERR_HIP, "flex_allreduce_staged_noalloc: cannot read the compute unit count: %s",
                              hipGetErrorString(e));
        g_num_cus[dev] = n;
        g_scratch_ptr[dev] = (unsigned char*)p;
    }
    *ptr = g_scratch_ptr[dev];
    *cus = g_num_cus[dev];
    return FLEX_OK;
}

}  // namespace

extern "C" int flex_allreduce_staged_noalloc(const void* const* rank_bufs, int nranks, int rank, void* out,
                                             size_t count, int dtype, int op, uint32_t staged_units,
                                             void* hip_stream) {
    const char* who = "flex_allreduce_staged_noalloc";
    const size_t es = flex::dtype_size(dtype);
    if (es == 0) return flex::fail(FLEX_ERR_UNSUPPORTED, "%s: unknown dtype %d", who, dtype);
    if (op != FLEX_SUM) return flex::fail(FLEX_ERR_UNSUPPORTED, "%s: unknown op %d", who, op);
    if (nranks < 1 || nranks > FLEX_MAX_RANKS || rank < 0 || rank >= nranks)
        return flex::fail(FLEX_ERR_INVALID_ARG, "%s: nranks %d / rank %d out of range", who, nranks, rank);
    if (staged_units > 10000) return flex::fail(FLEX_ERR_INVALID_ARG, "%s: staged_units %u exceed 10000", who, staged_units);
    if (!rank_bufs) return flex::fail(FLEX_ERR_INVALID_ARG, "%s: rank pointer array is NULL", who);
    if (count == 0) return FLEX_OK;
    if (!out || (uintptr_t)out % es) return flex::fail(FLEX_ERR_INVALID_ARG, "%s: out is NULL or misaligned", who);
    for (int r = 0; r < nranks; ++r)
        if (!rank_bufs[r] || (uintptr_t)rank_bufs[r] % es)
            return flex::fail(FLEX_ERR_INVALID_ARG, "%s: rank %d pointer is NULL or misaligned", who, r);

    // the cut of flex_allreduce_local at its default settings
    const uint64_t split = nranks > 1 ? flex::partition(count, staged_units, 10000, 2048, (64u << 10) / es) : count;
    const size_t part = (count - split) * es;             // staged bytes per peer
    const size_t stride = (part + 255) / 256 * 256;
    const size_t room = nranks > 1 ? kScratchBytes / (size_t)(nranks - 1) / 256 * 256 : 0;
    if (stride > room)
        return flex::fail(FLEX_ERR_INVALID_ARG,
                          "%s: the staged part is %zu bytes per peer, the built-in transit buffer of %zu bytes holds "
                          "at most %zu bytes for each of %d peers: lower staged_units or use flex_allreduce_local",
                          who, part, kScratchBytes, room, nranks - 1);

    unsigned char* transit = nullptr;
    int cus = 0;
    if (int st = scratch_for_current_device(&transit, &cus)) return st;

    hipStream_t stream = (hipStream_t)hip_stream;
    flex::LaunchShape reduce_shape{64, 1, 3, (uint32_t)cus, 0};
    reduce_shape.serial_min_tiles = 16u * (uint32_t)cus;
    reduce_shape.serial_min_inputs = 3;
    reduce_shape.serial_lds_bytes = 5632;  // the library's default occupancy cap for this schedule
    const flex::LaunchShape staged_reduce_shape{256, 1, 0, (uint32_t)cus, 0};
    const flex::LaunchShape staged_copy_shape{256, 2, 0, (uint32_t)cus, 0};

    auto launched = [&](int e) {
        return e == 0 ? FLEX_OK
                      : flex::fail(FLEX_ERR_HIP, "%s: kernel launch failed: %s", who, hipGetErrorString((hipError_t)e));
    };
    if (split > 0)
        if (int st = launched(flex::launch_reduce_n(rank_bufs, nranks, out, split, dtype, reduce_shape, stream))) return st;
    if (split == count) return FLEX_OK;

    // peers' parts -> transit buffer, then the reduce reads them from there in
    // rank order with the local rank's part read in place
    const void* src[FLEX_MAX_RANKS];
    void* dst[FLEX_MAX_RANKS];
    uint64_t nn[FLEX_MAX_RANKS];
    const void* in[FLEX_MAX_RANKS];
    int npeers = 0;
    for (int r = 0; r < nranks; ++r) {
        const char* piece = (const char*)rank_bufs[r] + split * es;
        if (r == rank) {
            in[r] = piece;
            continue;
        }
        src[npeers] = piece;
        dst[npeers] = transit + (size_t)npeers * stride;
        nn[npeers] = part;
        in[r] = dst[npeers];
        ++npeers;
    }
    if (int st = launched(flex::launch_gather_copy(src, dst, nn, npeers, staged_copy_shape, stream))) return st;
    return launched(flex::launch_reduce_n(in, nranks, (char*)out + split * es, count - split, dtype,
                                          staged_reduce_shape, stream));
}
