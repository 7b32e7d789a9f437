// Measurement only: what a plain streaming read reaches on this GPU with the request pattern of the MLA
// decode main kernel and no arithmetic.  It is the practical ceiling the benchmark reports beside the
// published peak ("roofline.achievable"): the decode kernel cannot stream faster than a kernel that
// does nothing but stream.  Not part of the product library and not declared in include/.
//
// Pattern, as in the main kernel: a persistent grid, one workgroup of four wavefronts per compute unit
// (the workgroup claims the same 150 KB of LDS, so no second one lands beside it); the buffer is cut
// into one contiguous range per wavefront; a wavefront keeps 36 requests of 1 KB (64 lanes x 16 bytes,
// fully sequential, non-temporal) in flight and re-issues each as soon as it has consumed it.
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int kDepth = 36;                  // 1 KB requests in flight per wavefront: one 32-row tile
constexpr int kWaves = 4;
constexpr int kLdsBytes = 150 * 1024;

__global__ void __launch_bounds__(kWaves * 64, 1) hbm_probe_read_kernel(const char *src, size_t bytes_per_wave, unsigned *sink) {
    extern __shared__ char smem[];
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    const char *base = src + ((size_t)blockIdx.x * kWaves + w) * bytes_per_wave + l * 16;
    const size_t rounds = bytes_per_wave / (kDepth * 1024);
    u32x4 v[kDepth];
#pragma unroll
    for (int i = 0; i < kDepth; ++i) v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(base + i * 1024));
    u32x4 acc = {0, 0, 0, 0};
    for (size_t r = 1; r < rounds; ++r) {
        const char *at = base + r * (kDepth * 1024);
#pragma unroll
        for (int i = 0; i < kDepth; ++i) {
            acc ^= v[i];
            v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(at + i * 1024));
        }
    }
#pragma unroll
    for (int i = 0; i < kDepth; ++i) acc ^= v[i];
    // the loads must not be optimised away: a result that depends on every byte, stored only if it
    // equals a value the caller's fill pattern never produces
    const unsigned x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    if (x == 0x9E3779B9u) {
        sink[0] = x;
        smem[threadIdx.x] = 1;
    }
}

}  // namespace

extern "C" {

// Launch the streaming read of `bytes` bytes at `src` (device, 16-byte aligned) over `workgroups`
// workgroups on `stream`; `sink` is 4 device bytes that are normally left untouched.  *bytes_read
// (host) receives the bytes the launch actually reads: `bytes` rounded down to a whole number of
// 36 KB rounds per wavefront.  Returns 0, or -1 on a bad argument or a failed launch.
int hbm_probe_read(const void *src, size_t bytes, int workgroups, void *sink, size_t *bytes_read, void *stream) {
    if (!src || !sink || !bytes_read || workgroups < 1 || workgroups > 65536 || (reinterpret_cast<uintptr_t>(src) & 15u)) return -1;
    const size_t per_wave = bytes / ((size_t)workgroups * kWaves) / (kDepth * 1024) * (kDepth * 1024);
    if (per_wave == 0) return -1;
    static bool attr_done = false;      // callers of this measurement aid are single-threaded
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(hbm_probe_read_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess)
            return -1;
        attr_done = true;
    }
    const char *s = static_cast<const char *>(src);
    size_t pw = per_wave;
    unsigned *sk = static_cast<unsigned *>(sink);
    void *args[] = {&s, &pw, &sk};
    if (hipLaunchKernel(reinterpret_cast<const void *>(hbm_probe_read_kernel), dim3(workgroups), dim3(kWaves * 64), args, kLdsBytes,
                        static_cast<hipStream_t>(stream)) != hipSuccess)
        return -1;
    *bytes_read = per_wave * (size_t)workgroups * kWaves;
    return 0;
}

}  // extern "C"
