// N-way rank-ordered reduction: the arithmetic a rank performs in the
// reduce-scatter half of the paper's ring AllReduce ("reduce sum computation",
// Limitations and Future Work), fused over all N contributions.
//
// Pure HBM streaming for gfx950: every lane issues one 16-byte load per input
// (a wavefront covers 1 KiB of each input contiguously) and
// the result leaves through one 16-byte store.  No LDS and no MFMA: 7 adds per
// 18 bytes.  Two load schedules: one puts all N loads of a tile in flight
// before the first add; the other ("serial") keeps ONE load in flight per
// wavefront - input r+1 is requested only after input r has arrived - and
// leaves the latency hiding to the 32 wavefronts a compute unit holds.
// On MI355X the serial schedule is the faster one by 3-7 % for messages of
// 4 MiB and more per rank (a wavefront's loads return in order, so eight
// outstanding loads to eight streams can hold each other up; measured, not
// derived).  Short messages, whose time is one wavefront's lifetime, are
// faster with all loads in flight; the launcher chooses by tile count.
//
// The sum is taken strictly in rank order in binary32, starting from rank 0's
// value, and rounded once to the element type; nothing here may be compiled
// with fast-math, reassociation or denormal flushing.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "flexlink_internal.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// The same vector at any element-aligned address.  gfx950 under ROCm serves
// vector loads from unaligned addresses (a load that straddles a line costs a
// second line access, nothing else), so an input need not share the output's
// offset within 16 bytes: only the stores are kept aligned.
typedef u32x4 u32x4_in __attribute__((aligned(2)));

struct ReduceArgs {
    const void* in[FLEX_MAX_RANKS];
    void* out;
    uint64_t head;   // leading elements handled one by one (until the output is tile-aligned)
    uint64_t nvec;   // 16-byte vectors in the aligned body
    uint64_t count;  // all elements
    uint32_t shift;  // only workgroups whose index is a multiple of 2^shift work
    // Launch dimensions as plain arguments: a kernel that reads blockDim / gridDim makes the
    // runtime fill in its hidden launch arguments, which costs 1 us of host time per launch.
    uint32_t nthreads;  // workgroup size
    uint32_t nblk;      // working workgroups (grid size >> shift)
};

template <bool NT>
__device__ __forceinline__ u32x4 load16(const u32x4_in* p) {
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

// bfloat16 is the upper half of a binary32: widening is a shift.
__device__ __forceinline__ float bf16_low_to_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_high_to_f32(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// binary32 -> bfloat16 bits, round to nearest even in integer arithmetic; a NaN
// keeps sign and upper payload and gets its quiet bit set.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    uint32_t rounded = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    uint32_t quiet = (u >> 16) | 0x0040u;
    return ((u & 0x7fffffffu) > 0x7f800000u) ? quiet : rounded;
}

// binary16 <-> binary32 through the hardware converters: the widening is exact,
// the narrowing rounds to nearest even (the default rounding mode) and keeps
// binary16 subnormals; a NaN stays a NaN.
__device__ __forceinline__ float f16_bits_to_f32(uint32_t h) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)h);
}
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f) {
    return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
}

// Element types (values of flex_dtype).
constexpr int kF32 = FLEX_F32, kBF16 = FLEX_BF16, kF16 = FLEX_F16;

template <int DT>
__device__ __forceinline__ float widen_low(uint32_t w) {
    return DT == kBF16 ? bf16_low_to_f32(w) : f16_bits_to_f32(w & 0xffffu);
}
template <int DT>
__device__ __forceinline__ float widen_high(uint32_t w) {
    return DT == kBF16 ? bf16_high_to_f32(w) : f16_bits_to_f32(w >> 16);
}
template <int DT>
__device__ __forceinline__ uint32_t narrow(float f) {
    return DT == kBF16 ? f32_to_bf16_bits(f) : f32_to_f16_bits(f);
}

// One 16-byte vector from each of N inputs -> one 16-byte result.
template <int N, int DT>
__device__ __forceinline__ u32x4 reduce_vectors(const u32x4 (&v)[N]) {
    u32x4 o;
    if (DT != kF32) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            float lo = widen_low<DT>(v[0][w]);
            float hi = widen_high<DT>(v[0][w]);
#pragma unroll
            for (int r = 1; r < N; ++r) {
                lo = lo + widen_low<DT>(v[r][w]);
                hi = hi + widen_high<DT>(v[r][w]);
            }
            o[w] = narrow<DT>(lo) | (narrow<DT>(hi) << 16);
        }
    } else {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            float acc = __uint_as_float(v[0][w]);
#pragma unroll
            for (int r = 1; r < N; ++r) acc = acc + __uint_as_float(v[r][w]);
            o[w] = __float_as_uint(acc);
        }
    }
    return o;
}

// Serial schedule: one 16-byte vector of every input, summed in rank order,
// with at most one load outstanding.  The index of the next load is passed
// through an empty asm statement together with the value just loaded, so the
// compiler can neither issue the next load early nor drop the dependence.
template <int N, int DT, bool LDNT>
__device__ __forceinline__ u32x4 reduce_serial(const u32x4_in* const (&in)[N], uint64_t idx) {
    constexpr int kAcc = DT == kF32 ? 4 : 8;
    float acc[kAcc];
    u32x4 v = load16<LDNT>(in[0] + idx);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        if (DT != kF32) {
            acc[2 * w] = widen_low<DT>(v[w]);
            acc[2 * w + 1] = widen_high<DT>(v[w]);
        } else {
            acc[w] = __uint_as_float(v[w]);
        }
    }
#pragma unroll
    for (int r = 1; r < N; ++r) {
        asm volatile("" : "+v"(idx) : "v"(v[0]));
        v = load16<LDNT>(in[r] + idx);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (DT != kF32) {
                acc[2 * w] = acc[2 * w] + widen_low<DT>(v[w]);
                acc[2 * w + 1] = acc[2 * w + 1] + widen_high<DT>(v[w]);
            } else {
                acc[w] = acc[w] + __uint_as_float(v[w]);
            }
        }
    }
    u32x4 o;
#pragma unroll
    for (int w = 0; w < 4; ++w)
        o[w] = DT != kF32 ? (narrow<DT>(acc[2 * w]) | (narrow<DT>(acc[2 * w + 1]) << 16)) : __float_as_uint(acc[w]);
    return o;
}

template <int N, int DT>
__device__ __forceinline__ void reduce_one_element(const ReduceArgs& a, uint64_t i) {
    if (DT != kF32) {
        float acc = widen_low<DT>(((const uint16_t*)a.in[0])[i]);
#pragma unroll
        for (int r = 1; r < N; ++r) acc = acc + widen_low<DT>(((const uint16_t*)a.in[r])[i]);
        ((uint16_t*)a.out)[i] = (uint16_t)narrow<DT>(acc);
    } else {
        float acc = ((const float*)a.in[0])[i];
#pragma unroll
        for (int r = 1; r < N; ++r) acc = acc + ((const float*)a.in[r])[i];
        ((float*)a.out)[i] = acc;
    }
}

template <int N, int DT, bool SERIAL, bool LDNT, bool STNT>
__global__ void reduce_n_kernel(ReduceArgs a) {
    constexpr uint32_t kElemSize = DT == kF32 ? 4 : 2;
    constexpr uint32_t kVecElems = 16 / kElemSize;
    const uint32_t tid = threadIdx.x;
    const uint32_t nthreads = a.nthreads;
    // Workgroups go to the 8 accelerator dies round-robin by index: with shift 3
    // the working ones all sit on one die.
    if (blockIdx.x & ((1u << a.shift) - 1u)) return;
    const uint32_t bid = blockIdx.x >> a.shift;
    const uint32_t nblk = a.nblk;
    const uint64_t ntiles = (a.nvec + nthreads - 1) / nthreads;  // one vector per thread and tile

    const u32x4_in* in[N];
#pragma unroll
    for (int r = 0; r < N; ++r)
        in[r] = (const u32x4_in*)((const char*)a.in[r] + a.head * kElemSize);
    u32x4* out = (u32x4*)((char*)a.out + a.head * kElemSize);

    for (uint64_t tile = bid; tile < ntiles; tile += nblk) {
        const uint64_t idx = tile * nthreads + tid;
        if (idx >= a.nvec) continue;  // ragged last tile
        if (SERIAL) {
            store16<STNT>(out + idx, reduce_serial<N, DT, LDNT>(in, idx));
        } else {
            u32x4 v[N];
#pragma unroll
            for (int r = 0; r < N; ++r) v[r] = load16<LDNT>(in[r] + idx);
            store16<STNT>(out + idx, reduce_vectors<N, DT>(v));
        }
    }

    // Elements outside the aligned body: [0, head) and [head + nvec*kVecElems, count).
    const uint64_t body_end = a.head + a.nvec * kVecElems;
    const uint64_t nscalar = a.head + (a.count - body_end);
    for (uint64_t k = (uint64_t)bid * nthreads + tid; k < nscalar; k += (uint64_t)nblk * nthreads) {
        const uint64_t i = k < a.head ? k : body_end + (k - a.head);
        reduce_one_element<N, DT>(a, i);
    }
}

// Streaming hints: 0 none, 1 non-temporal loads, 3 non-temporal loads and stores.
template <int N, int DT, bool SERIAL>
int launch_one(const ReduceArgs& a, uint32_t grid, uint32_t threads, uint32_t nt, uint32_t lds, hipStream_t stream) {
    switch (nt) {
        case 0: hipLaunchKernelGGL((reduce_n_kernel<N, DT, SERIAL, false, false>), dim3(grid), dim3(threads), lds, stream, a); break;
        case 1: hipLaunchKernelGGL((reduce_n_kernel<N, DT, SERIAL, true, false>), dim3(grid), dim3(threads), lds, stream, a); break;
        default: hipLaunchKernelGGL((reduce_n_kernel<N, DT, SERIAL, true, true>), dim3(grid), dim3(threads), lds, stream, a); break;
    }
    return (int)hipGetLastError();
}

template <int N, int DT>
int launch_n(const ReduceArgs& a, uint32_t grid, uint32_t threads, bool serial, uint32_t nt, uint32_t lds,
             hipStream_t stream) {
    return serial ? launch_one<N, DT, true>(a, grid, threads, nt, lds, stream)
                  : launch_one<N, DT, false>(a, grid, threads, nt, lds, stream);
}

template <int DT>
int launch_dtype(int n, const ReduceArgs& a, uint32_t grid, uint32_t threads, bool serial, uint32_t nt,
                 uint32_t lds, hipStream_t stream) {
    switch (n) {
        case 1: return launch_n<1, DT>(a, grid, threads, serial, nt, lds, stream);
        case 2: return launch_n<2, DT>(a, grid, threads, serial, nt, lds, stream);
        case 3: return launch_n<3, DT>(a, grid, threads, serial, nt, lds, stream);
        case 4: return launch_n<4, DT>(a, grid, threads, serial, nt, lds, stream);
        case 5: return launch_n<5, DT>(a, grid, threads, serial, nt, lds, stream);
        case 6: return launch_n<6, DT>(a, grid, threads, serial, nt, lds, stream);
        case 7: return launch_n<7, DT>(a, grid, threads, serial, nt, lds, stream);
        default: return launch_n<8, DT>(a, grid, threads, serial, nt, lds, stream);
    }
}

}  // namespace

namespace flex {

constexpr uintptr_t kTileBytes = 1024;  // one wavefront's 16-byte vectors

int launch_reduce_n(const void* const* in, int n, void* out, size_t count, int dtype,
                    const LaunchShape& shape, void* stream) {
    if (count == 0) return 0;
    const size_t esize = dtype_size(dtype);
    const size_t vec_elems = 16 / esize;
    ReduceArgs a;
    for (int r = 0; r < FLEX_MAX_RANKS; ++r) a.in[r] = r < n ? in[r] : nullptr;
    a.out = out;
    a.count = count;

    // The vector body starts where the output reaches a 1 KiB boundary, so
    // that every wavefront stores whole, tile-aligned lines (measured on
    // MI355X: a body that starts 16 or 64 bytes off a line is 15 % slower, one
    // that starts 256 bytes off a 1 KiB boundary 7 %).  Inputs that share the
    // output's offset within 1 KiB, the common case, come out aligned with it;
    // any other input is read through unaligned vector loads.
    uint64_t head = ((kTileBytes - ((uintptr_t)out & (kTileBytes - 1))) & (kTileBytes - 1)) / esize;
    if (head > count) head = count;
    a.head = head;
    a.nvec = (count - head) / vec_elems;

    const uint32_t threads = shape.threads;
    // The serial schedule pays N load latencies per tile: it wins once the
    // message keeps every wavefront slot of the chip busy several times over,
    // and loses on short messages whose time is one wavefront's lifetime.  With
    // two inputs it loses at every size (measured on MI355X, 2 x 32 MiB ... 2 x 1 GiB
    // of bf16: 1-5 % behind both loads in flight), which serial_min_inputs expresses.
    const bool serial = shape.serial_min_tiles && (uint32_t)n >= shape.serial_min_inputs &&
                        (a.nvec + 63) / 64 >= shape.serial_min_tiles;  // 1 KiB tiles
    const uint64_t ntiles = (a.nvec + threads - 1) / threads;
    const uint64_t nscalar = count - a.nvec * vec_elems;
    const uint64_t scalar_blocks = (nscalar + threads - 1) / threads;
    uint64_t grid = std::max(ntiles, std::min<uint64_t>(scalar_blocks, 8ull * shape.num_cus));
    if (shape.max_blocks && grid > shape.max_blocks) grid = shape.max_blocks;
    if (grid == 0) grid = 1;
    a.shift = shape.block_shift > 8 ? 8 : shape.block_shift;
    if (grid > (0x7fffffffull >> a.shift)) grid = 0x7fffffffull >> a.shift;
    a.nthreads = threads;
    a.nblk = (uint32_t)grid;
    grid <<= a.shift;

    // With one load in flight per wavefront a compute unit that holds its full 32
    // wavefronts runs 3-4 % slower than one that holds 25-31, once the launch is long
    // enough to reach a steady state and has four or more inputs (measured on MI355X:
    // +3 % at 8 x 256 MiB, +2 % at 4 x 256 MiB, +4 % at 4 x 1 GiB, but -1 to -2 % at
    // 3 x 128 and 3 x 256 MiB, -1 % with two inputs and -3 % at 8 x 32 MiB; the
    // all-in-flight schedule and the copy kernel lose with it at every size).  A small
    // LDS reservation per workgroup, which the kernel never touches, keeps the count
    // just below the limit for such launches: those that read at least
    // cap_min_tiles_per_cu tiles per compute unit.
    const uint64_t tiles_read = (uint64_t)(n + 1) * ((a.nvec + 63) / 64);
    const bool cap = serial && (uint32_t)n >= shape.cap_min_inputs &&
                     tiles_read >= (uint64_t)shape.cap_min_tiles_per_cu * shape.num_cus;
    const uint32_t lds = cap ? shape.serial_lds_bytes : shape.lds_bytes;
    hipStream_t s = (hipStream_t)stream;
    if (dtype == FLEX_BF16)
        return launch_dtype<kBF16>(n, a, (uint32_t)grid, threads, serial, shape.nontemporal, lds, s);
    if (dtype == FLEX_F16)
        return launch_dtype<kF16>(n, a, (uint32_t)grid, threads, serial, shape.nontemporal, lds, s);
    return launch_dtype<kF32>(n, a, (uint32_t)grid, threads, serial, shape.nontemporal, lds, s);
}

}  // namespace flex
