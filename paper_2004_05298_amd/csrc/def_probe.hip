// Streaming kernels of known traffic (include/def_probe.h): what a pure read, a pure
// write, a copy and an in-place update sustain in the launch shape of the streaming pass.
#include "def.h"
#include "def_probe.h"

#include <hip/hip_runtime.h>

typedef float v4f __attribute__((ext_vector_type(4)));

namespace {

// One workgroup covers THREADS * U float4 groups; lane t takes groups t, t + THREADS, ...
template <int KIND, int THREADS, int U>
__global__ __launch_bounds__(THREADS) void def_probe_kernel(const float *__restrict__ src, float *dst,
                                                            uint64_t groups, float value)
{
    const uint64_t first = (uint64_t)blockIdx.x * (THREADS * U) + threadIdx.x;
    v4f v[U];
    if constexpr (KIND != DEF_PROBE_WRITE) {
        const v4f *from = reinterpret_cast<const v4f *>(KIND == DEF_PROBE_UPDATE ? dst : src);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t q = first + (uint64_t)u * THREADS;
            v[u] = q < groups ? __builtin_nontemporal_load(from + q) : (v4f)(0.0f);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint64_t q = first + (uint64_t)u * THREADS;
        if (q >= groups) continue;
        if constexpr (KIND == DEF_PROBE_READ) {
            // keeps the load alive; the host passes a NaN, which no sum equals, so this never stores
            if (v[u][0] + v[u][1] + v[u][2] + v[u][3] == value && dst) dst[0] = value;
        } else if constexpr (KIND == DEF_PROBE_WRITE) {
            __builtin_nontemporal_store((v4f)(value), reinterpret_cast<v4f *>(dst) + q);
        } else if constexpr (KIND == DEF_PROBE_COPY) {
            __builtin_nontemporal_store(v[u], reinterpret_cast<v4f *>(dst) + q);
        } else {
            __builtin_nontemporal_store(v[u] * value, reinterpret_cast<v4f *>(dst) + q);
        }
    }
}

template <int KIND, int THREADS, int U>
void launch_probe(const float *src, float *dst, uint64_t groups, float value, uint32_t lds, hipStream_t st)
{
    const uint64_t per_block = (uint64_t)THREADS * U;
    const dim3 grid((uint32_t)((groups + per_block - 1) / per_block)), block(THREADS);
    def_probe_kernel<KIND, THREADS, U><<<grid, block, lds, st>>>(src, dst, groups, value);
}

template <int KIND>
bool launch_shape(uint32_t threads, uint32_t quads, const float *src, float *dst, uint64_t groups, float value,
                  uint32_t lds, hipStream_t st)
{
#define DEF_PROBE_CASE(T, Q) \
    if (threads == T && quads == Q) { launch_probe<KIND, T, Q>(src, dst, groups, value, lds, st); return true; }
    DEF_PROBE_CASE(64, 1) DEF_PROBE_CASE(64, 2) DEF_PROBE_CASE(64, 4)
    DEF_PROBE_CASE(256, 1) DEF_PROBE_CASE(256, 2) DEF_PROBE_CASE(256, 4)
#undef DEF_PROBE_CASE
    return false;
}

}  // namespace

extern "C" int def_probe_stream(int kind, const float *src, float *dst, uint64_t n, float value,
                                uint32_t threads, uint32_t quads, uint32_t lds_reserve, void *stream)
{
    if (kind < DEF_PROBE_READ || kind > DEF_PROBE_UPDATE) return DEF_EINVAL;
    if (n == 0 || n % 256 != 0 || n >= (1ull << 39) || lds_reserve > 65536) return DEF_EINVAL;
    const bool needs_src = kind == DEF_PROBE_READ || kind == DEF_PROBE_COPY;
    const bool needs_dst = kind != DEF_PROBE_READ;
    if ((needs_src && !src) || (needs_dst && !dst)) return DEF_EINVAL;
    if ((uintptr_t)src % 16 != 0 || (uintptr_t)dst % 16 != 0) return DEF_EINVAL;
    const uint64_t groups = n / 4;
    hipStream_t st = (hipStream_t)stream;
    bool known = false;
    switch (kind) {
    case DEF_PROBE_READ:
        known = launch_shape<DEF_PROBE_READ>(threads, quads, src, nullptr, groups, __builtin_nanf(""), lds_reserve, st);
        break;
    case DEF_PROBE_WRITE:
        known = launch_shape<DEF_PROBE_WRITE>(threads, quads, nullptr, dst, groups, value, lds_reserve, st);
        break;
    case DEF_PROBE_COPY:
        known = launch_shape<DEF_PROBE_COPY>(threads, quads, src, dst, groups, value, lds_reserve, st);
        break;
    default:
        known = launch_shape<DEF_PROBE_UPDATE>(threads, quads, nullptr, dst, groups, value, lds_reserve, st);
        break;
    }
    if (!known) return DEF_EINVAL;          // workgroup size or groups per lane not offered
    const hipError_t err = hipGetLastError();
    return err == hipSuccess ? DEF_OK : DEF_EHIP;
}
