// Measurement only: one LDS access pattern per launch, so that rocprofv3's SQ_LDS_BANK_CONFLICT and
// SQ_LDS_IDX_ACTIVE can be read pattern by pattern.  One wavefront repeats one LDS instruction, each lane
// at its own byte offset taken from a table, 4096 times.  The benchmark's --lds-probe mode feeds it the
// three access patterns of the MLA decode main kernel (K operand reads, transposing V^T reads, tile
// writes) for candidate row strides and token orders; the choice of the row stride of 1184 bytes rests
// on these readings.  Not part of the product library and not declared in include/.
#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) char lds_char;
constexpr int kIterations = 4096;
constexpr int kLdsBytes = 40 * 1024;

// op 0: ds_read_b128, 1: ds_write_b128, 2: ds_read_b64_tr_b16, 3: ds_write_b32
__global__ void __launch_bounds__(64) lds_probe_kernel(const int *offsets, int op, unsigned *sink) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int l = threadIdx.x;
    for (int i = l; i < kLdsBytes / 4; i += 64) reinterpret_cast<unsigned *>(smem)[i] = i;
    __syncthreads();
    char *at = smem + offsets[l];
    u32x4 acc = {0, 0, 0, 0};
    if (op == 0) {
        for (int it = 0; it < kIterations; ++it) acc ^= *reinterpret_cast<volatile u32x4 *>(at);
    } else if (op == 1) {
        for (int it = 0; it < kIterations; ++it) {
            *reinterpret_cast<volatile u32x4 *>(at) = acc;
            acc[0] += 1;
        }
    } else if (op == 3) {
        for (int it = 0; it < kIterations; ++it) {
            *reinterpret_cast<volatile unsigned *>(at) = acc[0];
            acc[0] += 1;
        }
    } else {
        for (int it = 0; it < kIterations; ++it) {
            const i16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)(lds_char *)at);
            asm volatile("" ::"v"(v));
            acc[0] ^= (unsigned)v[0];
        }
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9E3779B9u) sink[0] = 1;    // keeps the loop alive; never true in practice
}

}  // namespace

extern "C" {

// One launch of the pattern: `offsets` is a device array of 64 byte offsets (each a multiple of 8, the
// access inside the first 40 KB of LDS: checked by the caller, which builds the table), `op` selects the
// instruction (0 ds_read_b128, 1 ds_write_b128, 2 ds_read_b64_tr_b16, 3 ds_write_b32), `sink` 4 device bytes.
// Returns 0, or -1 on a bad argument or a failed launch.
int lds_probe_run(const int *offsets, int op, void *sink, void *stream) {
    if (!offsets || !sink || op < 0 || op > 3) return -1;
    static bool attr_done = false;      // callers of this measurement aid are single-threaded
    if (!attr_done) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(lds_probe_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess)
            return -1;
        attr_done = true;
    }
    unsigned *sk = static_cast<unsigned *>(sink);
    void *args[] = {&offsets, &op, &sk};
    return hipLaunchKernel(reinterpret_cast<const void *>(lds_probe_kernel), dim3(1), dim3(64), args, kLdsBytes,
                           static_cast<hipStream_t>(stream)) == hipSuccess ? 0 : -1;
}

}  // extern "C"
