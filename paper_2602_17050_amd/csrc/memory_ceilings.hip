// Measures, on the GPU it runs on, the memory-system ceilings that bound the MPZCH remap path:
// the path is a hash-table probe, i.e. independent random accesses of 4..128 bytes, so what limits
// it is the rate of random requests the memory system sustains, not streaming bandwidth.
// Stand-alone tool (no dependency on the library): prints one line per access pattern.
//
//   memory_ceilings [slots]      slots: size of the int64 array that is probed (default 1e9 = 8 GB)
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>
#include <cstdlib>

#define CK(x)                                                                              \
    do {                                                                                   \
        hipError_t e_ = (x);                                                               \
        if (e_ != hipSuccess) {                                                            \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);   \
            return 1;                                                                      \
        }                                                                                  \
    } while (0)

__device__ __forceinline__ uint64_t mix64(uint64_t x)
{
    uint64_t z = x + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__global__ void k_copy(const uint4 *a, uint4 *b, uint64_t n)
{
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x) b[i] = a[i];
}

// one 8-byte load per thread at a uniformly random slot
__global__ void k_gather8(const long long *t, uint64_t n, uint64_t ops, long long *sink)
{
    long long a = 0;
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < ops; i += (uint64_t)gridDim.x * blockDim.x)
        a += t[__umul64hi(mix64(i), n)];
    if (a == 0x1234567) sink[0] = a;
}

// 16 lanes read one random 128-byte line (aligned) or 16 consecutive slots from a random slot (unaligned)
template <bool ALIGNED>
__global__ void k_line(const long long *t, uint64_t n, uint64_t ops, long long *sink)
{
    long long a = 0;
    const uint64_t tid = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    const uint64_t groups = ((uint64_t)gridDim.x * blockDim.x) >> 4;
    const int r = tid & 15;
    for (uint64_t i = tid >> 4; i < ops; i += groups * 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint64_t j = i + u * groups;
            if (j < ops) {
                uint64_t s = __umul64hi(mix64(j), n - 32);
                if (ALIGNED) s &= ~15ull;
                a += t[s + r];
            }
        }
    }
    if (a == 0x1234567) sink[0] = a;
}

// As k_line<true>, but the accesses are issued in address order at the granularity of `buckets` equal
// parts of the array: access j falls into part j * buckets / ops, at a random line inside it (what a
// batch looks like after its positions were bucketed by the top bits of their home slot).
__global__ void k_line_bucketed(const long long *t, uint64_t n, uint64_t ops, uint64_t buckets, long long *sink)
{
    long long a = 0;
    const uint64_t tid = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    const uint64_t groups = ((uint64_t)gridDim.x * blockDim.x) >> 4;
    const int r = tid & 15;
    const uint64_t part = (n - 32) / buckets;
    const double scale = (double)buckets / (double)ops;
    // a workgroup walks a contiguous range of accesses, so that neighbouring workgroups stay in neighbouring parts
    const uint64_t per_group = (ops + groups - 1) / groups;
    const uint64_t j0 = (tid >> 4) * per_group;
    for (uint64_t k = 0; k < per_group; k += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint64_t j = j0 + k + u;
            if (k + u < per_group && j < ops) {
                uint64_t b = (uint64_t)((double)j * scale);     // the part, up to rounding at its borders
                if (b >= buckets) b = buckets - 1;
                uint64_t s = b * part + __umul64hi(mix64(j), part);
                s &= ~15ull;
                a += t[s + r];
            }
        }
    }
    if (a == 0x1234567) sink[0] = a;
}

// 4-byte stores in the same bucketed order
__global__ void k_store4_bucketed(int *t, uint64_t n, uint64_t ops, uint64_t buckets)
{
    const uint64_t tid = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    const uint64_t threads = (uint64_t)gridDim.x * blockDim.x;
    const uint64_t part = n / buckets;
    const double scale = (double)buckets / (double)ops;
    const uint64_t per_wave = (ops + threads - 1) / threads * 64;
    const uint64_t j0 = (tid >> 6) * per_wave + (tid & 63);
    for (uint64_t k = 0; k < per_wave; k += 64) {
        const uint64_t j = j0 + k;
        if (j < ops) {
            uint64_t b = (uint64_t)((double)j * scale);
            if (b >= buckets) b = buckets - 1;
            t[b * part + __umul64hi(mix64(j), part)] = 7;
        }
    }
}

// The metadata refresh as part of the line that was fetched for the identities: 16 lanes read one random
// aligned 128-byte line, then one of them stores 4 bytes -- into the SAME line (an interleaved
// identities + metadata layout) or into a second array at the matching place (the two-tensor layout).
// NT: the line is read with non-temporal loads.
template <bool SAME, bool NT = false>
__global__ void k_line_then_store4(long long *t, int *m, uint64_t n, uint64_t ops, long long *sink)
{
    long long a = 0;
    const uint64_t tid = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    const uint64_t groups = ((uint64_t)gridDim.x * blockDim.x) >> 4;
    const int r = tid & 15;
    for (uint64_t i = tid >> 4; i < ops; i += groups * 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint64_t j = i + u * groups;
            if (j < ops) {
                const uint64_t s = __umul64hi(mix64(j), n - 32) & ~15ull;
                const long long v = NT ? __builtin_nontemporal_load(&t[s + r]) : t[s + r];
                a += v;
                if (r == 15) {
                    // the store depends on the value read, as a refresh depends on the match
                    if (SAME) reinterpret_cast<int *>(&t[s + 15])[1] = (int)v | 7;
                    else m[s + 15] = (int)v | 7;
                }
            }
        }
    }
    if (a == 0x1234567) sink[0] = a;
}

__global__ void k_store4(int *t, uint64_t n, uint64_t ops)
{
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < ops; i += (uint64_t)gridDim.x * blockDim.x)
        t[__umul64hi(mix64(i), n)] = 7;
}

// LANES consecutive lanes write one random aligned chunk of LANES * 16 bytes (16 .. 128 bytes)
template <int LANES>
__global__ void k_store_chunk(uint4 *t, uint64_t n16, uint64_t ops)
{
    const uint64_t tid = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    const uint64_t groups = ((uint64_t)gridDim.x * blockDim.x) / LANES;
    const int r = tid % LANES;
    for (uint64_t i = tid / LANES; i < ops; i += groups) {
        const uint64_t c = __umul64hi(mix64(i), n16 / LANES);
        t[c * LANES + r] = make_uint4(7u, 7u, 7u, 7u);
    }
}

// a 4-byte atomic max whose result is not used, at a random slot
__global__ void k_atomic_max4(int *t, uint64_t n, uint64_t ops)
{
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < ops; i += (uint64_t)gridDim.x * blockDim.x)
        (void)__hip_atomic_fetch_max(&t[__umul64hi(mix64(i), n)], 7, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// the word is read first, then written (the line is in the cache when the store arrives)
__global__ void k_load_store4(int *t, uint64_t n, uint64_t ops)
{
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < ops; i += (uint64_t)gridDim.x * blockDim.x) {
        int *p = &t[__umul64hi(mix64(i), n)];
        const int v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *p = v | 7;
    }
}

__global__ void k_store4_nt(int *t, uint64_t n, uint64_t ops)
{
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < ops; i += (uint64_t)gridDim.x * blockDim.x)
        __builtin_nontemporal_store(7, &t[__umul64hi(mix64(i), n)]);
}

__global__ void k_atomic_min(long long *t, uint64_t n, uint64_t ops, long long *sink)
{
    long long a = 0;
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < ops; i += (uint64_t)gridDim.x * blockDim.x)
        a += __hip_atomic_fetch_min(&t[__umul64hi(mix64(i), n)], (long long)(i | 0x4000000000000000ull), __ATOMIC_RELAXED,
                                    __HIP_MEMORY_SCOPE_AGENT);
    if (a == 0x1234567) sink[0] = a;
}

// one atomic per wavefront, all on ONE address (what a shared list cursor costs)
__global__ void k_same_address(unsigned long long *c, unsigned long long *sink)
{
    unsigned long long b = 0;
    if ((threadIdx.x & 63) == 0) b = atomicAdd(c, 64ull);
    if (b == 0x1234567) sink[0] = b;
}

int main(int argc, char **argv)
{
    // a multiple of 1024 slots keeps both halves of the array 16-byte aligned
    const uint64_t n = (argc > 1 ? std::strtoull(argv[1], nullptr, 10) : 1000000000ull) & ~1023ull;
    if (n < 65536 || n > (1ull << 34)) {
        std::printf("slots must lie in [65536, 2^34]\n");
        return 1;
    }
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    long long *t;
    int *m;
    unsigned long long *c;
    CK(hipMalloc(&t, n * 8));
    CK(hipMalloc(&m, n * 4));
    CK(hipMalloc(&c, 4096));
    CK(hipMemset(t, 0x7f, n * 8));
    CK(hipMemset(m, 0, n * 4));
    CK(hipMemset(c, 0, 4096));
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    std::printf("device: %s, %d compute units; probed array: %llu int64 slots (%.1f GB)\n", prop.name,
                prop.multiProcessorCount, (unsigned long long)n, n * 8 / 1e9);
    float ms = 0.f;
    auto report = [&](const char *name, double ops, double bytes_per_op) {
        std::printf("%-58s %8.3f ms %9.2f G ops/s %9.1f GB/s\n", name, ms, ops / ms / 1e6, ops * bytes_per_op / ms / 1e6);
        std::fflush(stdout);
    };
#define TIME(launch)                          \
    launch;                                   \
    CK(hipDeviceSynchronize());               \
    CK(hipEventRecord(e0));                   \
    launch;                                   \
    CK(hipEventRecord(e1));                   \
    CK(hipEventSynchronize(e1));              \
    CK(hipEventElapsedTime(&ms, e0, e1));
    const uint64_t ops = 64000000ull;
    // the copy reads the first half of the array and writes the second: at most 2 GiB, never more than half
    uint64_t copy_bytes = n * 4 < (1ull << 31) ? n * 4 : (1ull << 31);
    copy_bytes &= ~15ull;
    const uint64_t cn = copy_bytes / 16;
    TIME((k_copy<<<8192, 256>>>((const uint4 *)t, (uint4 *)(t + (n / 2)), cn)));
    std::printf("streaming copy moves %.3f GiB each way\n", copy_bytes / 1073741824.0);
    report("streaming copy (read + written)", (double)cn, 32.0);
    TIME((k_gather8<<<8192, 256>>>(t, n, ops, (long long *)c + 8)));
    report("random 8-byte loads (one per lane)", (double)ops, 8.0);
    TIME((k_line<true><<<8192, 256>>>(t, n, ops, (long long *)c + 8)));
    report("random aligned 128-byte lines (16 lanes each)", (double)ops, 128.0);
    TIME((k_line<false><<<8192, 256>>>(t, n, ops, (long long *)c + 8)));
    report("random unaligned 128-byte windows (16 lanes each)", (double)ops, 128.0);
    for (uint64_t buckets : {2048ull, 65536ull, 2097152ull}) {
        char name[96];
        TIME((k_line_bucketed<<<8192, 256>>>(t, n, ops, buckets, (long long *)c + 8)));
        std::snprintf(name, sizeof name, "aligned 128-byte lines in address order, %llu parts", (unsigned long long)buckets);
        report(name, (double)ops, 128.0);
    }
    TIME((k_line_then_store4<false><<<8192, 256>>>(t, m, n, ops, (long long *)c + 8)));
    report("random line read + 4-byte store into a second array", (double)ops, 132.0);
    TIME((k_line_then_store4<true><<<8192, 256>>>(t, m, n, ops, (long long *)c + 8)));
    report("random line read + 4-byte store into the same line", (double)ops, 132.0);
    TIME((k_line_then_store4<false, true><<<8192, 256>>>(t, m, n, ops, (long long *)c + 8)));
    report("non-temporal line read + 4-byte store into a second array", (double)ops, 132.0);
    TIME((k_line_then_store4<true, true><<<8192, 256>>>(t, m, n, ops, (long long *)c + 8)));
    report("non-temporal line read + 4-byte store into the same line", (double)ops, 132.0);
    TIME((k_store4<<<8192, 256>>>(m, n, ops)));
    report("random 4-byte stores (one per lane)", (double)ops, 4.0);
    for (uint64_t buckets : {2048ull, 65536ull, 2097152ull}) {
        char name[96];
        TIME((k_store4_bucketed<<<8192, 256>>>(m, n, ops, buckets)));
        std::snprintf(name, sizeof name, "4-byte stores in address order, %llu parts", (unsigned long long)buckets);
        report(name, (double)ops, 4.0);
    }
    TIME((k_store4_nt<<<8192, 256>>>(m, n, ops)));
    report("random 4-byte non-temporal stores (one per lane)", (double)ops, 4.0);
    TIME((k_load_store4<<<8192, 256>>>(m, n, ops)));
    report("random 4-byte load, then store to the same word", (double)ops, 4.0);
    TIME((k_atomic_max4<<<8192, 256>>>(m, n, ops)));
    report("random 4-byte atomic max, result unused (one per lane)", (double)ops, 4.0);
    TIME((k_store_chunk<1><<<8192, 256>>>((uint4 *)m, n / 4, ops)));
    report("random aligned 16-byte stores (one lane each)", (double)ops, 16.0);
    TIME((k_store_chunk<2><<<8192, 256>>>((uint4 *)m, n / 4, ops)));
    report("random aligned 32-byte stores (2 lanes each)", (double)ops, 32.0);
    TIME((k_store_chunk<4><<<8192, 256>>>((uint4 *)m, n / 4, ops)));
    report("random aligned 64-byte stores (4 lanes each)", (double)ops, 64.0);
    TIME((k_store_chunk<8><<<8192, 256>>>((uint4 *)m, n / 4, ops)));
    report("random aligned 128-byte stores (8 lanes each)", (double)ops, 128.0);
    TIME((k_atomic_min<<<8192, 256>>>(t, n, ops / 4, (long long *)c + 8)));
    report("random 64-bit atomic min with return (one per lane)", (double)ops / 4, 8.0);
    TIME((k_same_address<<<16384, 256>>>(c, c + 8)));
    report("atomic add on ONE address, one per wavefront (65536)", 65536.0, 8.0);
    return 0;
}
