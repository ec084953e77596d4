// Measurement aids of bench.py, built into their own small library (libagentsam_bench.so) and not part of
// the product ABI.
//   bench_stream_read_probe  a plain streaming read of a device buffer, i.e. the rate the memory system delivers
//                            to a kernel that does nothing else.  Same access shape as the attention kernels:
//                            every wavefront reads whole 16 KB tiles with 16-byte non-temporal loads, 1 KB
//                            contiguous per instruction.
//   bench_paged_read_probe   the loads of the narrow attention kernel on a batch of equally long sessions and
//                            nothing else: the same grid (one workgroup per compute unit), the same assignment of
//                            (session, kv head) streams to workgroups, every tile's K and V rows found through the
//                            block table, two tiles per wavefront in flight; no staging, no arithmetic.
// The benchmark quotes spec_verify_attn against both, next to the published HBM peak.
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

// K, V: [num_pages][Hkv][P][D] bf16; bt: [B][max_pages]; every session has tiles_per_session 32-position tiles.
// Workgroup w reads streams w*spw .. w*spw+spw-1 (stream = session * Hkv + kv head) one after the other.
__global__ __launch_bounds__(256) void paged_read_kernel(const char *__restrict__ K, const char *__restrict__ V,
                                                         const int *__restrict__ bt, int max_pages,
                                                         long long num_pages, int B, int Hkv,
                                                         int P, int D, int tiles_per_session, int spw,
                                                         u32x4 *__restrict__ sink) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const size_t row_bytes = (size_t)D * 2, tile_bytes = 32 * row_bytes;
    const int loads = (int)(tile_bytes / 1024);              // 1 KB per load instruction: 8 for D = 128
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (int h = 0; h < spw; ++h) {
        const int s = (int)blockIdx.x * spw + h;
        if (s >= B * Hkv) break;
        const int b = s / Hkv, kvh = s % Hkv;
        const int *row = bt + (size_t)b * max_pages;
        for (int t = wave; t < tiles_per_session; t += 8) {   // tiles t and t + 4 together
            u32x4 v[32];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int tt = t + 4 * u < tiles_per_session ? t + 4 * u : t;
                const int pos0 = tt * 32;
                int page = row[pos0 / P];
                if (page < 0 || page >= num_pages) page = 0;  // (never the case for the benchmark's tables)
                const size_t off = (((size_t)page * Hkv + kvh) * P + pos0 % P) * row_bytes;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const size_t o = off + (size_t)(i < loads ? i : 0) * 1024;
                    v[u * 16 + 2 * i] = __builtin_nontemporal_load((const u32x4 *)(K + o) + lane);
                    v[u * 16 + 2 * i + 1] = __builtin_nontemporal_load((const u32x4 *)(V + o) + lane);
                }
            }
#pragma unroll
            for (int i = 0; i < 32; ++i) acc ^= v[i];
        }
    }
    if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u && acc.z == 0x0badf00du) sink[0] = acc;
}
}  // namespace

// Reads the K and V rows of B sessions of tiles_per_session * 32 positions each through the block table, once, with
// 256 workgroups (device pointers; the caches hold num_pages pages; a block-table entry outside them reads page 0).
// 0 on success, -1 null pointer, -2 bad shape (P not a multiple of 32, D not 64 or 128, sessions longer than the
// table), -6 launch failed.
extern "C" int bench_paged_read_probe(const void *k_cache, const void *v_cache, const int *block_table, int max_pages,
                                      long long num_pages, int B, int Hkv, int P, int D, int tiles_per_session,
                                      void *sink16, void *stream) {
    if (!k_cache || !v_cache || !block_table || !sink16) return -1;
    if (B < 1 || Hkv < 1 || num_pages < 1 || P < 32 || P % 32 != 0 || (D != 64 && D != 128) || tiles_per_session < 1 ||
        (long long)tiles_per_session * 32 > (long long)max_pages * P)
        return -2;
    constexpr int kWgs = 256;
    const int spw = (B * Hkv + kWgs - 1) / kWgs;
    paged_read_kernel<<<dim3(kWgs), dim3(256), 0, (hipStream_t)stream>>>((const char *)k_cache, (const char *)v_cache,
                                                                         block_table, max_pages, num_pages, B, Hkv,
                                                                         P, D, tiles_per_session, spw, (u32x4 *)sink16);
    return hipPeekAtLastError() == hipSuccess ? 0 : -6;
}

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
