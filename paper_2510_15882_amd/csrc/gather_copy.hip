// Chunked gather/copy: the data movement a rank performs in the all-gather half
// of the paper's ring collectives (Evaluation, "End-to-End Performance": N-1
// steps, each placing one rank's slice at its rank offset), done for all N
// slices in a single launch.
//
// Pure HBM streaming for gfx950: blockIdx.y selects the slice, lanes move
// 16-byte vectors so that a wavefront covers 1 KiB contiguously, UNROLL loads
// are in flight per lane before the first store.  Bytes are never interpreted;
// source and destination may sit at any byte addresses.
#include <hip/hip_runtime.h>

#include "flexlink_internal.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// The same vector at any byte address: gfx950 under ROCm serves vector loads
// from unaligned addresses (a load that straddles a line costs a second line
// access), so source and destination need not agree within 16 bytes.  Only
// the stores are kept aligned.
typedef u32x4 u32x4_src __attribute__((aligned(1)));

struct CopyArgs {
    const void* src[FLEX_MAX_RANKS];
    void* dst[FLEX_MAX_RANKS];
    uint64_t bytes[FLEX_MAX_RANKS];
    uint32_t shift;  // only workgroups whose x index is a multiple of 2^shift work
    // Launch dimensions as plain arguments: a kernel that reads blockDim / gridDim makes the
    // runtime fill in its hidden launch arguments, which costs 1 us of host time per launch.
    uint32_t nthreads;  // workgroup size
    uint32_t nblk;      // working workgroups along x (grid size >> shift)
};

template <bool NT>
__device__ __forceinline__ u32x4 load16(const u32x4_src* p) {
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}

template <bool NT>
__device__ __forceinline__ void store16(u32x4* p, u32x4 v) {
    if (NT)
        __builtin_nontemporal_store(v, p);
    else
        *p = v;
}

template <int UNROLL, bool LDNT, bool STNT>
__global__ void gather_copy_kernel(CopyArgs a) {
    const int r = blockIdx.y;
    const char* s = (const char*)a.src[r];
    char* d = (char*)a.dst[r];
    const uint64_t bytes = a.bytes[r];
    if (s == d || bytes == 0) return;  // slice already in place
    // Workgroups go to the 8 accelerator dies round-robin by linear index, and
    // the grid's x size is a multiple of 2^shift: with shift 3 the working ones all sit
    // on one die.
    if (blockIdx.x & ((1u << a.shift) - 1u)) return;
    const uint32_t bid = blockIdx.x >> a.shift;
    const uint32_t nblk = a.nblk;

    const uint32_t tid = threadIdx.x;
    const uint32_t nthreads = a.nthreads;
    // body from where the destination reaches a 1 KiB boundary: every wavefront
    // then stores whole, tile-aligned lines (a source at the same offset within
    // 1 KiB, the common case, is aligned there too)
    uint64_t head = (1024 - ((uintptr_t)d & 1023)) & 1023;
    if (head > bytes) head = bytes;
    const uint64_t nvec = (bytes - head) / 16;
    const u32x4_src* in = (const u32x4_src*)(s + head);
    u32x4* out = (u32x4*)(d + head);
    const uint64_t tile_vecs = (uint64_t)nthreads * UNROLL;
    const uint64_t ntiles = (nvec + tile_vecs - 1) / tile_vecs;

    for (uint64_t tile = bid; tile < ntiles; tile += nblk) {
        const uint64_t first = tile * tile_vecs;
        if (first + tile_vecs <= nvec) {
            u32x4 v[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) v[u] = load16<LDNT>(in + first + (uint64_t)u * nthreads + tid);
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) store16<STNT>(out + first + (uint64_t)u * nthreads + tid, v[u]);
        } else {
            for (int u = 0; u < UNROLL; ++u) {
                const uint64_t idx = first + (uint64_t)u * nthreads + tid;
                if (idx < nvec) store16<STNT>(out + idx, load16<LDNT>(in + idx));
            }
        }
    }

    // bytes outside the aligned body (at most 1023 in front, 15 behind)
    const uint64_t body_end = head + nvec * 16;
    const uint64_t nloose = head + (bytes - body_end);
    if (bid == 0) {
        for (uint64_t k = tid; k < nloose; k += nthreads) {
            const uint64_t i = k < head ? k : body_end + (k - head);
            d[i] = s[i];
        }
    }
}

// Streaming hints: 0 none, 1 non-temporal loads, 3 non-temporal loads and stores.
template <int UNROLL>
int launch_one(const CopyArgs& a, dim3 grid, uint32_t threads, uint32_t nt, uint32_t lds, hipStream_t stream) {
    switch (nt) {
        case 0: hipLaunchKernelGGL((gather_copy_kernel<UNROLL, false, false>), grid, dim3(threads), lds, stream, a); break;
        case 1: hipLaunchKernelGGL((gather_copy_kernel<UNROLL, true, false>), grid, dim3(threads), lds, stream, a); break;
        default: hipLaunchKernelGGL((gather_copy_kernel<UNROLL, true, true>), grid, dim3(threads), lds, stream, a); break;
    }
    return (int)hipGetLastError();
}

}  // namespace

namespace flex {

int launch_gather_copy(const void* const* src, void* const* dst, const uint64_t* bytes, int n,
                       const LaunchShape& shape, void* stream) {
    CopyArgs a;
    uint64_t longest = 0;
    for (int r = 0; r < FLEX_MAX_RANKS; ++r) {
        a.src[r] = r < n ? src[r] : nullptr;
        a.dst[r] = r < n ? dst[r] : nullptr;
        a.bytes[r] = r < n ? bytes[r] : 0;
        if (r < n && src[r] != dst[r] && bytes[r] > longest) longest = bytes[r];
    }
    if (longest == 0) return 0;

    const uint32_t threads = shape.threads;
    const uint32_t unroll = shape.unroll == 2 || shape.unroll == 4 || shape.unroll == 6 ? shape.unroll : 1;
    const uint64_t tile_bytes = (uint64_t)threads * unroll * 16;
    uint64_t gx = (longest + tile_bytes - 1) / tile_bytes;
    if (shape.max_blocks) {
        uint64_t per_slice = shape.max_blocks / (uint32_t)n;
        if (per_slice == 0) per_slice = 1;
        if (gx > per_slice) gx = per_slice;
    }
    if (gx == 0) gx = 1;
    a.shift = shape.block_shift > 8 ? 8 : shape.block_shift;
    if (gx > (0x7fffffffull >> a.shift)) gx = 0x7fffffffull >> a.shift;
    a.nthreads = threads;
    a.nblk = (uint32_t)gx;
    gx <<= a.shift;
    dim3 grid((uint32_t)gx, (uint32_t)n, 1);
    hipStream_t s = (hipStream_t)stream;
    switch (unroll) {
        case 2: return launch_one<2>(a, grid, threads, shape.nontemporal, shape.lds_bytes, s);
        case 4: return launch_one<4>(a, grid, threads, shape.nontemporal, shape.lds_bytes, s);
        case 6: return launch_one<6>(a, grid, threads, shape.nontemporal, shape.lds_bytes, s);
        default: return launch_one<1>(a, grid, threads, shape.nontemporal, shape.lds_bytes, s);
    }
}

}  // namespace flex
