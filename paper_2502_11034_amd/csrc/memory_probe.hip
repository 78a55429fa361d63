// Measurement tool, not part of the library: what the memory system gives a streaming kernel shaped like the
// update kernel (work items of 4096 elements, 128-bit streaming accesses, four per lane and array in flight), for a
// given mix of arrays read and arrays written in place.  The update kernel of the AdaGC step reads g, theta, m, v
// and writes theta, m, v (Alg. 1's last four statements): 4 reads + 3 in-place writes.
// Built as a library of its own (libadagc_probe.so); driven by memory_probe.py.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kMaxArrays = 8;
constexpr int kItemElems = 4096;           // 256 lanes x 4 vectors x 4 elements

struct Arrays {
    f32x4* base[kMaxArrays];
};

// Arrays 0 .. NR-1 are read, arrays 0 .. NW-1 written (in place where NW <= NR; the rest written only).
template <int NR, int NW>
__global__ __launch_bounds__(256) void stream_kernel(Arrays a, uint32_t n_items)
{
    const size_t item = blockIdx.x;
    if (item >= n_items) return;
    const size_t first = item * (kItemElems / 4) + threadIdx.x;
    f32x4 x[4][NR > 0 ? NR : 1];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int s = 0; s < NR; ++s) x[u][s] = __builtin_nontemporal_load(a.base[s] + first + (size_t)u * 256);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        f32x4 v = {1.f, 2.f, 3.f, 4.f};
#pragma unroll
        for (int s = 0; s < NR; ++s) v += x[u][s];
#pragma unroll
        for (int s = 0; s < NW; ++s) __builtin_nontemporal_store(v * (float)(s + 1), a.base[s] + first + (size_t)u * 256);
        if constexpr (NW == 0) {
            // keeps the loads alive: never true for the driver's data (zeros and small sums)
            if (v.x == -1.2345e30f) a.base[0][first + (size_t)u * 256] = v;
        }
    }
}

template <int NR, int NW>
hipError_t launch(const Arrays& a, uint32_t n_items, hipStream_t stream)
{
    stream_kernel<NR, NW><<<dim3(n_items), dim3(256), 0, stream>>>(a, n_items);
    return hipGetLastError();
}

}  // namespace

// One launch over `elems` elements (a multiple of 4096, at most 2^31 items) of each array, on `stream`.
//   arrays   HOST array of max(n_read, n_write) DEVICE pointers, fp32, 16-byte aligned, each `elems` long
// Supported mixes (n_read, n_write): (4,0) (1,0) (0,4) (0,1) (4,3) (1,1) (2,1).  Returns 0, or -1 for anything else.
extern "C" int adagc_probe_stream(void* const* arrays, int n_read, int n_write, int64_t elems, void* stream)
{
    if (!arrays || elems <= 0 || elems % kItemElems != 0 || elems / kItemElems > 0x7FFFFFFF) return -1;
    const int n = n_read > n_write ? n_read : n_write;
    if (n < 1 || n > kMaxArrays) return -1;
    Arrays a{};
    for (int i = 0; i < n; ++i) {
        if (!arrays[i] || (reinterpret_cast<uintptr_t>(arrays[i]) & 15u)) return -1;
        a.base[i] = static_cast<f32x4*>(arrays[i]);
    }
    const uint32_t items = (uint32_t)(elems / kItemElems);
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = hipErrorInvalidValue;
    if (n_read == 4 && n_write == 0) e = launch<4, 0>(a, items, s);
    else if (n_read == 1 && n_write == 0) e = launch<1, 0>(a, items, s);
    else if (n_read == 0 && n_write == 4) e = launch<0, 4>(a, items, s);
    else if (n_read == 0 && n_write == 1) e = launch<0, 1>(a, items, s);
    else if (n_read == 4 && n_write == 3) e = launch<4, 3>(a, items, s);
    else if (n_read == 1 && n_write == 1) e = launch<1, 1>(a, items, s);
    else if (n_read == 2 && n_write == 1) e = launch<2, 1>(a, items, s);
    return e == hipSuccess ? 0 : -1;
}
