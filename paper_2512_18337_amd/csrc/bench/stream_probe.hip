// Measurement aid of bench.py, built into its own small library (libagentsam_bench.so) and not part of
// the product ABI: a plain streaming read of a device buffer, i.e. the rate the memory system delivers
// to a kernel that does nothing else.  The benchmark quotes spec_verify_attn against it next to the
// published HBM peak.  Same access shape as the attention kernels: every wavefront reads whole 16 KB
// tiles with 16-byte non-temporal loads, 1 KB contiguous per instruction.
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace {
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4 *__restrict__ p, size_t tiles_per_wg,
                                                          u32x4 *__restrict__ sink) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const u32x4 *base = p + (size_t)blockIdx.x * tiles_per_wg * 1024;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (size_t t = wave; t < tiles_per_wg; t += 4) {
        u32x4 v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = __builtin_nontemporal_load(base + t * 1024 + i * 64 + lane);
#pragma unroll
        for (int i = 0; i < 16; ++i) acc ^= v[i];
    }
    // never true for the benchmark's buffer; keeps the loads alive
    if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u && acc.z == 0x0badf00du) sink[0] = acc;
}
}  // namespace

// Reads buf[0 .. bytes rounded down to 16 MiB) once with 1024 workgroups (device pointers; sink16 = 16
// writable bytes, normally left untouched).  0 on success, -1 null pointer, -2 fewer than 16 MiB, -6 launch failed.
extern "C" int bench_stream_read_probe(const void *buf, size_t bytes, void *sink16, void *stream) {
    if (!buf || !sink16) return -1;
    constexpr int kWgs = 1024;
    const size_t tiles_per_wg = bytes / 16384 / kWgs;
    if (tiles_per_wg == 0) return -2;
    stream_read_kernel<<<dim3(kWgs), dim3(256), 0, (hipStream_t)stream>>>((const u32x4 *)buf, tiles_per_wg, (u32x4 *)sink16);
    return hipPeekAtLastError() == hipSuccess ? 0 : -6;
}
