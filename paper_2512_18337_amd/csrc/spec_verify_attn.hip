// spec_verify_attn: attention of the verification pass (Alg. 4, "Validate with main LLM"):
// the 1+k query rows of every session (base token + k drafts) against that session's paged
// KV cache, causal among the new rows, grouped-query heads.
//
// The work is a stream over the KV cache: every K/V byte is needed once per (session, kv head)
// and is used by all G*(1+k) query rows that share that kv head, so the kernel is bound by HBM
// bandwidth and is organised around reading each byte exactly once:
//
//   - one workgroup per (session, kv head, row group, KV chunk); its 4 wavefronts take the
//     chunk's 32-position tiles round-robin, so the workgroup streams one contiguous region;
//   - a wavefront loads its next tile (16-byte coalesced loads) while it computes the current
//     one, stages it in its own LDS region, and runs two MFMA contractions on it with the
//     query rows packed as (head-in-group, row) into 16-row tiles:
//         S^T = K . Q^T   (positions x rows, contraction over head_dim)
//         O^T += V^T . P^T (head_dim x rows, contraction over the tile's positions)
//     The S^T accumulator layout (4 consecutive positions per lane for one row) is exactly the
//     B-operand layout of the second contraction once the positions of a tile are enumerated in
//     that order, so P never leaves registers; V is transposed on its way out of LDS;
//   - online softmax in fp32 (base-2 exponent, running maximum and sum per row);
//   - the 4 wavefronts merge through LDS; a session with one chunk is written directly, longer
//     ones leave (O, m, l) partials in the workspace for the log-sum-exp merge kernel.
//
// The fp32 storage type runs through a plain (non-MFMA) kernel with the same chunking.
#include <hip/hip_bf16.h>

#include "common.h"

namespace agentsam {
int64_t option_attn_v_mode();
}

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;          // finite stand-in for -inf in running maxima
constexpr int kTile = 32;                    // KV positions per wavefront step
constexpr int kWaves = 4;
constexpr int kRowsPerGroup = 48;            // 3 MFMA row tiles of 16 per wavefront
constexpr int kF32Chunk = 256;               // KV positions per workgroup of the fp32 kernel
constexpr int kF32MaxR = 32;

struct AttnParams {
    const void *q, *kc, *vc;
    const int32_t *bt, *seq;
    void *out;
    float *ws;
    int B, R, Hq, Hkv, G, P, max_pages;
    int64_t num_pages;
    float scale_log2;        // scale * log2(e)
    int chunk;               // KV positions per workgroup
    int nchunks_max;         // grid extent over chunks
    int rows;                // G*R packed rows per kv head
    int n_rg;                // row groups of kRowsPerGroup rows
    int rows_pad;            // rows per workspace record
    int out_bf16;
};

// workspace record of one (session, head group, chunk): o[rows_pad][D], m[rows_pad], l[rows_pad]
__device__ __forceinline__ int64_t ws_record_floats(int rows_pad, int D) { return (int64_t)rows_pad * (D + 2); }

__device__ __forceinline__ void store_out(void *out, int64_t idx, float4 v, int out_bf16) {
    if (out_bf16) {
        __hip_bfloat16 *o = (__hip_bfloat16 *)out + idx;
        o[0] = __float2bfloat16(v.x); o[1] = __float2bfloat16(v.y);
        o[2] = __float2bfloat16(v.z); o[3] = __float2bfloat16(v.w);
    } else {
        *(float4 *)((float *)out + idx) = v;
    }
}

// ------------------------------------------------------------------------------------------
// bf16 MFMA kernel
// ------------------------------------------------------------------------------------------
template <int D>
struct Bf16Cfg {
    static constexpr int kKStr = D * 2 + 16;                 // LDS row strides in bytes (padded against
    static constexpr int kVStr = D * 2 + 32;                 // bank conflicts of the two read patterns)
    static constexpr int kWaveBytes = kTile * (kKStr + kVStr);
    static constexpr int kOStr = D + 4;                      // floats
    static constexpr int kStageBytes = kWaves * kWaveBytes;
    static constexpr int kMergeBytes = kRowsPerGroup * kOStr * 4;
    static constexpr int kSmemBytes = (kStageBytes > kMergeBytes ? kStageBytes : kMergeBytes);
    static constexpr int kLoads = D / 16;                    // 16-byte loads per lane per tile, for K and for V
};

__device__ __forceinline__ void wave_lds_fence() {
    // LDS operations of one wavefront execute in order; this only stops the compiler from moving
    // LDS accesses of different lanes across the point where a tile changes hands.
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <int D, int MT, int VMODE>
__global__ __launch_bounds__(256) void attn_bf16_kernel(const AttnParams p) {
    using C = Bf16Cfg<D>;
    __shared__ __align__(16) char smem[C::kSmemBytes];
    __shared__ float red_m[kWaves * kRowsPerGroup];
    __shared__ float red_l[kWaves * kRowsPerGroup];

    const int chunk = blockIdx.x;
    const int kvh = blockIdx.y / p.n_rg;
    const int rg = blockIdx.y % p.n_rg;
    const int b = blockIdx.z;
    const int S = min(p.seq[b], p.max_pages * p.P);      // never index past the block table
    const int c0 = chunk * p.chunk;
    if (c0 >= S) return;                                     // uniform over the workgroup
    const int c1 = min(S, c0 + p.chunk);
    const int ntiles = (c1 - c0 + kTile - 1) / kTile;
    const int nchunks_b = (S + p.chunk - 1) / p.chunk;

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int n = lane & 15;                                 // MFMA column / A-row index
    const int g = lane >> 4;                                 // MFMA k-group
    const int R = p.R;

    char *Ks = smem + wave * C::kWaveBytes;
    char *Vs = Ks + kTile * C::kKStr;

    const __hip_bfloat16 *qg = (const __hip_bfloat16 *)p.q;
    const __hip_bfloat16 *kg = (const __hip_bfloat16 *)p.kc;
    const __hip_bfloat16 *vg = (const __hip_bfloat16 *)p.vc;

    // ---- Q fragments (B operand of S^T = K.Q^T): column n = packed row, 8 consecutive d per lane
    bf16x8 qf[MT][D / 32];
    int irow[MT];                                            // query row index (0..R-1) of this lane's column
#pragma unroll
    for (int rt = 0; rt < MT; ++rt) {
        const int pr = rg * kRowsPerGroup + rt * 16 + n;
        const bool live = pr < p.rows;
        const int hh = live ? pr / R : 0;
        const int i = live ? pr % R : R - 1;
        irow[rt] = i;
        const __hip_bfloat16 *src = qg + (((int64_t)b * R + i) * p.Hq + (int64_t)kvh * p.G + hh) * D;
#pragma unroll
        for (int ks = 0; ks < D / 32; ++ks) {
            s16x8 raw = {0, 0, 0, 0, 0, 0, 0, 0};
            if (live) raw = *(const s16x8 *)(src + ks * 32 + g * 8);
            qf[rt][ks] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    f32x4 oacc[D / 16][MT];
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt)
#pragma unroll
        for (int rt = 0; rt < MT; ++rt) oacc[dt][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run[MT], l_part[MT];
#pragma unroll
    for (int rt = 0; rt < MT; ++rt) { m_run[rt] = kNegBig; l_part[rt] = 0.f; }

    // ---- tile loads: lane -> (row, 16-byte column) so that one instruction reads 1 KB contiguous
    constexpr int kLanesPerRow = D / 8;
    constexpr int kRowsPerLoad = 64 / kLanesPerRow;
    const int ld_row = lane / kLanesPerRow;
    const int ld_col = lane % kLanesPerRow;
    uint4 kreg[C::kLoads], vreg[C::kLoads];

    auto issue_loads = [&](int t) {
        const int pos0 = c0 + t * kTile;
        const int page = p.bt[(int64_t)b * p.max_pages + pos0 / p.P];
        const bool page_ok = (unsigned)page < (unsigned long long)p.num_pages && page >= 0;
        const int64_t base = (((int64_t)(page_ok ? page : 0) * p.Hkv + kvh) * p.P + (pos0 % p.P)) * D;
#pragma unroll
        for (int i = 0; i < C::kLoads; ++i) {
            const int row = i * kRowsPerLoad + ld_row;
            const bool ok = page_ok && (pos0 + row < S);
            const int64_t off = base + (int64_t)row * D + ld_col * 8;
            kreg[i] = ok ? *(const uint4 *)(kg + off) : uint4{0u, 0u, 0u, 0u};
            vreg[i] = ok ? *(const uint4 *)(vg + off) : uint4{0u, 0u, 0u, 0u};
        }
    };

    int t = wave;
    if (t < ntiles) issue_loads(t);
    for (; t < ntiles; t += kWaves) {
        // hand the prefetched tile to LDS
#pragma unroll
        for (int i = 0; i < C::kLoads; ++i) {
            const int row = i * kRowsPerLoad + ld_row;
            *(uint4 *)(Ks + row * C::kKStr + ld_col * 16) = kreg[i];
            *(uint4 *)(Vs + row * C::kVStr + ld_col * 16) = vreg[i];
        }
        wave_lds_fence();
        if (t + kWaves < ntiles) issue_loads(t + kWaves);

        const int pos0 = c0 + t * kTile;

        // ---- S^T = K . Q^T : two 16-position tiles x MT row tiles
        f32x4 sacc[2][MT];
#pragma unroll
        for (int pt = 0; pt < 2; ++pt)
#pragma unroll
            for (int rt = 0; rt < MT; ++rt) sacc[pt][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < D / 32; ++ks) {
            bf16x8 kf[2];
#pragma unroll
            for (int pt = 0; pt < 2; ++pt)
                kf[pt] = *(const bf16x8 *)(Ks + (pt * 16 + n) * C::kKStr + (ks * 32 + g * 8) * 2);
#pragma unroll
            for (int pt = 0; pt < 2; ++pt)
#pragma unroll
                for (int rt = 0; rt < MT; ++rt)
                    sacc[pt][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[pt], qf[rt][ks], sacc[pt][rt], 0, 0, 0);
        }

        // ---- online softmax; lane holds, for column n of each row tile, positions pt*16 + 4g + r
        const bool need_mask = pos0 + kTile > S - R;         // tile touches the new rows or the ragged end
        bf16x8 pf[MT];
#pragma unroll
        for (int rt = 0; rt < MT; ++rt) {
            float sv[8];
#pragma unroll
            for (int pt = 0; pt < 2; ++pt)
#pragma unroll
                for (int r = 0; r < 4; ++r) sv[pt * 4 + r] = sacc[pt][rt][r] * p.scale_log2;
            bool allowed[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) allowed[j] = true;
            if (need_mask) {
                const int limit = S - R + irow[rt];          // last visible position of this row
#pragma unroll
                for (int pt = 0; pt < 2; ++pt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int pos = pos0 + pt * 16 + 4 * g + r;
                        allowed[pt * 4 + r] = pos <= limit;
                        if (!allowed[pt * 4 + r]) sv[pt * 4 + r] = kNegBig;
                    }
            }
            float mx = sv[0];
#pragma unroll
            for (int j = 1; j < 8; ++j) mx = fmaxf(mx, sv[j]);
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run[rt], mx);
            const float alpha = __builtin_amdgcn_exp2f(m_run[rt] - m_new);
            m_run[rt] = m_new;
            float ps[8];
            float psum = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                float e = __builtin_amdgcn_exp2f(sv[j] - m_new);
                if (need_mask && !allowed[j]) e = 0.f;
                ps[j] = e;
                psum += e;
            }
            l_part[rt] = l_part[rt] * alpha + psum;
            bf16x8 pk;
#pragma unroll
            for (int j = 0; j < 8; ++j) pk[j] = (__bf16)ps[j];
            pf[rt] = pk;
#pragma unroll
            for (int dt = 0; dt < D / 16; ++dt) oacc[dt][rt] *= alpha;
        }

        // ---- O^T += V^T . P^T ; k-slot 8g+j <-> position (j<4 ? 4g+j : 16+4g+j-4)
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) {
            bf16x8 vf;
            if (VMODE == 1) {
                // LDS transpose read (per 16 lanes): lane r supplies the 8-byte chunk (position r/4,
                // d-chunk r%4); lane i receives element i%4 of the chunks of lanes i/4, 4+i/4, 8+i/4,
                // 12+i/4, i.e. d = 16*dt + i at 4 consecutive positions
                const int bq = n & 3, jq = n >> 2;
                const char *a0 = Vs + (4 * g + jq) * C::kVStr + (dt * 16 + 4 * bq) * 2;
                const char *a1 = a0 + 16 * C::kVStr;
                s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)a0);
                s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)a1);
                s16x8 cat = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                vf = __builtin_bit_cast(bf16x8, cat);
            } else {
                s16x8 cat;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int pos = (j < 4) ? (4 * g + j) : (16 + 4 * g + j - 4);
                    cat[j] = *(const short *)(Vs + pos * C::kVStr + (dt * 16 + n) * 2);
                }
                vf = __builtin_bit_cast(bf16x8, cat);
            }
#pragma unroll
            for (int rt = 0; rt < MT; ++rt)
                oacc[dt][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[rt], oacc[dt][rt], 0, 0, 0);
        }
        wave_lds_fence();
    }

    // ---- merge the 4 wavefronts through LDS
    float l_tot[MT];
#pragma unroll
    for (int rt = 0; rt < MT; ++rt) {
        float l = l_part[rt];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        l_tot[rt] = l;
    }
    __syncthreads();                                         // staging LDS is free from here on
    if (g == 0) {
#pragma unroll
        for (int rt = 0; rt < MT; ++rt) {
            red_m[wave * kRowsPerGroup + rt * 16 + n] = m_run[rt];
            red_l[wave * kRowsPerGroup + rt * 16 + n] = l_tot[rt];
        }
    }
    __syncthreads();
    float my_scale[MT], M_all[MT], L_all[MT];
#pragma unroll
    for (int rt = 0; rt < MT; ++rt) {
        const int row = rt * 16 + n;
        float M = red_m[row];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) M = fmaxf(M, red_m[w * kRowsPerGroup + row]);
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w)
            L += red_l[w * kRowsPerGroup + row] * __builtin_amdgcn_exp2f(red_m[w * kRowsPerGroup + row] - M);
        M_all[rt] = M;
        L_all[rt] = L;
        my_scale[rt] = __builtin_amdgcn_exp2f(m_run[rt] - M);
    }
    float *Osum = (float *)smem;
    for (int w = 0; w < kWaves; ++w) {
        if (wave == w) {
#pragma unroll
            for (int rt = 0; rt < MT; ++rt)
#pragma unroll
                for (int dt = 0; dt < D / 16; ++dt) {
                    float4 *dst = (float4 *)(Osum + (rt * 16 + n) * C::kOStr + dt * 16 + 4 * g);
                    const f32x4 a = oacc[dt][rt] * my_scale[rt];
                    float4 v{a[0], a[1], a[2], a[3]};
                    if (w > 0) { const float4 o = *dst; v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w; }
                    *dst = v;
                }
        }
        __syncthreads();
    }
    // red_m/red_l of wavefront 0 now carry the merged maximum and sum (every wavefront computed the
    // same values; reads of the per-wavefront entries finished before the barriers above)
    if (wave == 0 && g == 0) {
#pragma unroll
        for (int rt = 0; rt < MT; ++rt) { red_m[rt * 16 + n] = M_all[rt]; red_l[rt * 16 + n] = L_all[rt]; }
    }
    __syncthreads();

    const int rows_here = min(MT * 16, p.rows - rg * kRowsPerGroup);
    if (nchunks_b == 1) {
        for (int idx = tid; idx < rows_here * (D / 4); idx += 256) {
            const int row = idx / (D / 4), c4 = idx % (D / 4);
            const int pr = rg * kRowsPerGroup + row;
            const int hh = pr / R, i = pr % R;
            const float inv = 1.0f / red_l[row];
            float4 v = *(const float4 *)(Osum + row * C::kOStr + c4 * 4);
            v.x *= inv; v.y *= inv; v.z *= inv; v.w *= inv;
            const int64_t o = (((int64_t)b * R + i) * p.Hq + (int64_t)kvh * p.G + hh) * D + c4 * 4;
            store_out(p.out, o, v, p.out_bf16);
        }
    } else {
        const int64_t rec = ((int64_t)b * p.Hkv + kvh) * p.nchunks_max + chunk;
        float *wo = p.ws + rec * ws_record_floats(p.rows_pad, D);
        float *wm = wo + (int64_t)p.rows_pad * D;
        float *wl = wm + p.rows_pad;
        for (int idx = tid; idx < rows_here * (D / 4); idx += 256) {
            const int row = idx / (D / 4), c4 = idx % (D / 4);
            const int pr = rg * kRowsPerGroup + row;
            *(float4 *)(wo + (int64_t)pr * D + c4 * 4) = *(const float4 *)(Osum + row * C::kOStr + c4 * 4);
        }
        if (tid < rows_here) {
            wm[rg * kRowsPerGroup + tid] = red_m[tid];
            wl[rg * kRowsPerGroup + tid] = red_l[tid];
        }
    }
}

// ------------------------------------------------------------------------------------------
// log-sum-exp merge of the chunk partials (sessions with more than one chunk)
//   out = sum_c 2^(m_c - M) o_c / sum_c 2^(m_c - M) l_c ,  M = max_c m_c
// grid (heads_outer, B); heads_outer = Hkv (bf16 path, rows = G*R packed) or Hq (fp32 path, rows = R)
// ------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void attn_merge_kernel(const AttnParams p, int heads_outer, int G_eff) {
    const int ho = blockIdx.x, b = blockIdx.y;
    const int S = min(p.seq[b], p.max_pages * p.P);      // never index past the block table
    const int nchunks_b = (S + p.chunk - 1) / p.chunk;
    if (nchunks_b <= 1) return;
    const int rows = G_eff * p.R;
    const int64_t recf = ws_record_floats(p.rows_pad, D);
    const float *base = p.ws + ((int64_t)b * heads_outer + ho) * p.nchunks_max * recf;
    for (int idx = threadIdx.x; idx < rows * (D / 4); idx += 256) {
        const int pr = idx / (D / 4), c4 = idx % (D / 4);
        float M = kNegBig;
        for (int c = 0; c < nchunks_b; ++c) M = fmaxf(M, base[c * recf + (int64_t)p.rows_pad * D + pr]);
        float L = 0.f;
        float4 acc{0.f, 0.f, 0.f, 0.f};
        for (int c = 0; c < nchunks_b; ++c) {
            const float *rec = base + c * recf;
            const float w = exp2f(rec[(int64_t)p.rows_pad * D + pr] - M);
            L += w * rec[(int64_t)p.rows_pad * D + p.rows_pad + pr];
            const float4 o = *(const float4 *)(rec + (int64_t)pr * D + c4 * 4);
            acc.x += w * o.x; acc.y += w * o.y; acc.z += w * o.z; acc.w += w * o.w;
        }
        const float inv = 1.0f / L;
        acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
        const int hh = pr / p.R, i = pr % p.R;
        const int64_t o = (((int64_t)b * p.R + i) * p.Hq + (int64_t)ho * G_eff + hh) * D + c4 * 4;
        store_out(p.out, o, acc, p.out_bf16);
    }
}

// ------------------------------------------------------------------------------------------
// fp32 storage: plain three-pass kernel per (chunk, query head, session)
// ------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void attn_f32_kernel(const AttnParams p) {
    __shared__ float qs[kF32MaxR][D];
    __shared__ float sc[kF32MaxR][kF32Chunk];
    __shared__ int64_t voff[kF32Chunk];
    __shared__ float row_m[kF32MaxR], row_l[kF32MaxR];

    const int chunk = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int S = min(p.seq[b], p.max_pages * p.P);      // never index past the block table
    const int c0 = chunk * p.chunk;
    if (c0 >= S) return;
    const int c1 = min(S, c0 + p.chunk);
    const int npos = c1 - c0;
    const int nchunks_b = (S + p.chunk - 1) / p.chunk;
    const int R = p.R, kvh = h / p.G;
    const int tid = threadIdx.x;
    const float *qg = (const float *)p.q;
    const float *kg = (const float *)p.kc;
    const float *vg = (const float *)p.vc;

    for (int idx = tid; idx < R * D; idx += 256) {
        const int i = idx / D, d = idx % D;
        qs[i][d] = qg[(((int64_t)b * R + i) * p.Hq + h) * D + d];
    }
    __syncthreads();

    // pass 1: scores (base-2 exponent domain), one position per thread
    if (tid < npos) {
        const int pos = c0 + tid;
        const int page = p.bt[(int64_t)b * p.max_pages + pos / p.P];
        const bool ok = page >= 0 && (int64_t)page < p.num_pages;
        const int64_t off = (((int64_t)(ok ? page : 0) * p.Hkv + kvh) * p.P + pos % p.P) * D;
        voff[tid] = ok ? off : -1;
        for (int i = 0; i < R; ++i) {
            float dot = 0.f;
            if (ok) {
#pragma unroll 4
                for (int d = 0; d < D; d += 4) {
                    const float4 kk = *(const float4 *)(kg + off + d);
                    dot = fmaf(qs[i][d], kk.x, dot); dot = fmaf(qs[i][d + 1], kk.y, dot);
                    dot = fmaf(qs[i][d + 2], kk.z, dot); dot = fmaf(qs[i][d + 3], kk.w, dot);
                }
            }
            sc[i][tid] = (pos <= S - R + i) ? dot * p.scale_log2 : -INFINITY;
        }
    }
    __syncthreads();

    // pass 2: per-row maximum and weights, one wavefront per row
    const int wave = tid >> 6, lane = tid & 63;
    for (int i = wave; i < R; i += 4) {
        float mx = -INFINITY;
        for (int t = lane; t < npos; t += 64) mx = fmaxf(mx, sc[i][t]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
        const float m = (mx == -INFINITY) ? kNegBig : mx;    // a row that sees nothing in this chunk
        float sum = 0.f;
        for (int t = lane; t < npos; t += 64) {
            const float e = exp2f(sc[i][t] - m);             // -inf -> 0
            sc[i][t] = e;
            sum += e;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
        if (lane == 0) { row_m[i] = m; row_l[i] = sum; }
    }
    __syncthreads();

    // pass 3: o[i][d] = sum_t w[i][t] * V[t][d]
    constexpr int kSlots = 256 / D;
    const int d = tid % D, slot = tid / D;
    float *wo = nullptr, *wm = nullptr, *wl = nullptr;
    if (nchunks_b > 1) {
        const int64_t rec = ((int64_t)b * p.Hq + h) * p.nchunks_max + chunk;
        wo = p.ws + rec * ws_record_floats(p.rows_pad, D);
        wm = wo + (int64_t)p.rows_pad * D;
        wl = wm + p.rows_pad;
    }
    for (int i = slot; i < R; i += kSlots) {
        float acc = 0.f;
        for (int t = 0; t < npos; ++t) {
            const int64_t off = voff[t];
            const float v = (off >= 0) ? vg[off + d] : 0.f;
            acc = fmaf(sc[i][t], v, acc);
        }
        if (nchunks_b > 1) {
            wo[(int64_t)i * D + d] = acc;
            if (d == 0) { wm[i] = row_m[i]; wl[i] = row_l[i]; }
        } else {
            const float r = acc / row_l[i];
            const int64_t o = (((int64_t)b * R + i) * p.Hq + h) * D + d;
            if (p.out_bf16) ((__hip_bfloat16 *)p.out)[o] = __float2bfloat16(r);
            else ((float *)p.out)[o] = r;
        }
    }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
struct Plan {
    int chunk, nchunks_max, n_rg, rows_pad, heads_outer;
    size_t ws_bytes;
};

int make_plan(int B, int R, int Hq, int Hkv, int D, int page_size, int max_pages, int dtype, Plan *pl) {
    if (B < 0 || R < 1 || Hq < 1 || Hkv < 1 || page_size < 1 || max_pages < 1) return AGENTSAM_ERR_ARG;
    if (Hq % Hkv != 0) return AGENTSAM_ERR_ARG;
    if (D != 64 && D != 128) return AGENTSAM_ERR_UNSUPPORTED;
    if (dtype != AGENTSAM_F32 && dtype != AGENTSAM_BF16) return AGENTSAM_ERR_UNSUPPORTED;
    const int64_t smax = (int64_t)max_pages * page_size;
    if (smax > 0x7fffff00ll) return AGENTSAM_ERR_ARG;
    const int G = Hq / Hkv;
    const int64_t opt = agentsam::option_attn_kv_chunk();
    if (dtype == AGENTSAM_F32) {
        if (R > kF32MaxR) return AGENTSAM_ERR_UNSUPPORTED;
        pl->chunk = kF32Chunk;                               // fixed: the score tile lives in LDS
        pl->n_rg = 1;
        pl->rows_pad = R;
        pl->heads_outer = Hq;
    } else {
        if (page_size % kTile != 0) return AGENTSAM_ERR_UNSUPPORTED;
        const int rows = G * R;
        if (rows > 4 * kRowsPerGroup) return AGENTSAM_ERR_UNSUPPORTED;
        pl->n_rg = (rows + kRowsPerGroup - 1) / kRowsPerGroup;
        pl->rows_pad = pl->n_rg * kRowsPerGroup;
        pl->heads_outer = Hkv;
        int64_t chunk = opt;
        if (chunk == 0) {
            // aim at ~2048 workgroups (8 per compute unit) when the sequences are long enough
            const int64_t pairs = (int64_t)B * Hkv * pl->n_rg;
            chunk = smax * (pairs > 0 ? pairs : 1) / 2048;
            chunk = (chunk + 127) / 128 * 128;
            if (chunk < 1024) chunk = 1024;
            if (chunk > 8192) chunk = 8192;
        }
        pl->chunk = (int)chunk;
    }
    pl->nchunks_max = (int)((smax + pl->chunk - 1) / pl->chunk);
    pl->ws_bytes = (size_t)B * pl->heads_outer * pl->nchunks_max * (size_t)pl->rows_pad * (D + 2) * sizeof(float);
    if (pl->nchunks_max <= 1) pl->ws_bytes = 0;
    return AGENTSAM_OK;
}

template <int D, int VMODE>
void launch_bf16(const AttnParams &p, dim3 grid, hipStream_t st) {
    const int rows_last = p.rows - (p.n_rg - 1) * kRowsPerGroup;   // all groups but the last are full
    // one instantiation per row-tile count of the (possibly partial) last group would need two
    // launches; a partially filled group simply carries dead rows instead
    (void)rows_last;
    const int mt = (p.n_rg > 1) ? 3 : (p.rows + 15) / 16;
    if (mt == 1) hipLaunchKernelGGL((attn_bf16_kernel<D, 1, VMODE>), grid, dim3(256), 0, st, p);
    else if (mt == 2) hipLaunchKernelGGL((attn_bf16_kernel<D, 2, VMODE>), grid, dim3(256), 0, st, p);
    else hipLaunchKernelGGL((attn_bf16_kernel<D, 3, VMODE>), grid, dim3(256), 0, st, p);
}

}  // namespace

extern "C" int spec_verify_attn_workspace(int32_t B, int32_t R, int32_t Hq, int32_t Hkv, int32_t D,
                                          int32_t page_size, int32_t max_pages, int32_t dtype, size_t *bytes) {
    if (!bytes) return AGENTSAM_ERR_NULL;
    Plan pl;
    const int rc = make_plan(B, R, Hq, Hkv, D, page_size, max_pages, dtype, &pl);
    if (rc) return rc;
    *bytes = pl.ws_bytes;
    return AGENTSAM_OK;
}

extern "C" int spec_verify_attn(const void *q, const void *k_cache, const void *v_cache,
                                const int32_t *block_table, int32_t max_pages, const int32_t *seq_lens,
                                int32_t B, int32_t R, int32_t Hq, int32_t Hkv, int32_t D, int32_t page_size,
                                int64_t num_pages, float scale, int32_t dtype, int32_t out_dtype,
                                void *out, void *workspace, size_t workspace_bytes, void *stream) {
    Plan pl;
    const int rc = make_plan(B, R, Hq, Hkv, D, page_size, max_pages, dtype, &pl);
    if (rc) return rc;
    if (!(scale > 0.f) || num_pages < 0) return AGENTSAM_ERR_ARG;
    if (out_dtype != AGENTSAM_F32 && out_dtype != AGENTSAM_BF16) return AGENTSAM_ERR_UNSUPPORTED;
    if (B == 0) return AGENTSAM_OK;
    if (!q || !k_cache || !v_cache || !block_table || !seq_lens || !out) return AGENTSAM_ERR_NULL;
    if (pl.ws_bytes > 0 && !workspace) return AGENTSAM_ERR_NULL;
    if (workspace_bytes < pl.ws_bytes) return AGENTSAM_ERR_WORKSPACE;
    if ((int64_t)B * pl.heads_outer * pl.n_rg > 65535ll * 65535ll) return AGENTSAM_ERR_ARG;

    AttnParams p;
    p.q = q; p.kc = k_cache; p.vc = v_cache; p.bt = block_table; p.seq = seq_lens; p.out = out;
    p.ws = (float *)workspace;
    p.B = B; p.R = R; p.Hq = Hq; p.Hkv = Hkv; p.G = Hq / Hkv; p.P = page_size; p.max_pages = max_pages;
    p.num_pages = num_pages;
    p.scale_log2 = scale * kLog2e;
    p.chunk = pl.chunk; p.nchunks_max = pl.nchunks_max;
    p.rows = p.G * R; p.n_rg = pl.n_rg; p.rows_pad = pl.rows_pad;
    p.out_bf16 = (out_dtype == AGENTSAM_BF16);
    hipStream_t st = (hipStream_t)stream;

    if (dtype == AGENTSAM_F32) {
        dim3 grid((unsigned)pl.nchunks_max, (unsigned)Hq, (unsigned)B);
        if (D == 64) hipLaunchKernelGGL(attn_f32_kernel<64>, grid, dim3(256), 0, st, p);
        else hipLaunchKernelGGL(attn_f32_kernel<128>, grid, dim3(256), 0, st, p);
        AGENTSAM_LAUNCH_CHECK();
        if (pl.nchunks_max > 1) {
            dim3 mg((unsigned)Hq, (unsigned)B);
            if (D == 64) hipLaunchKernelGGL(attn_merge_kernel<64>, mg, dim3(256), 0, st, p, (int)Hq, 1);
            else hipLaunchKernelGGL(attn_merge_kernel<128>, mg, dim3(256), 0, st, p, (int)Hq, 1);
            AGENTSAM_LAUNCH_CHECK();
        }
        return AGENTSAM_OK;
    }

    dim3 grid((unsigned)pl.nchunks_max, (unsigned)(Hkv * pl.n_rg), (unsigned)B);
    const bool tr = agentsam::option_attn_v_mode() == 1;
    if (D == 64) { if (tr) launch_bf16<64, 1>(p, grid, st); else launch_bf16<64, 0>(p, grid, st); }
    else { if (tr) launch_bf16<128, 1>(p, grid, st); else launch_bf16<128, 0>(p, grid, st); }
    AGENTSAM_LAUNCH_CHECK();
    if (pl.nchunks_max > 1) {
        dim3 mg((unsigned)Hkv, (unsigned)B);
        if (D == 64) hipLaunchKernelGGL(attn_merge_kernel<64>, mg, dim3(256), 0, st, p, (int)Hkv, p.G);
        else hipLaunchKernelGGL(attn_merge_kernel<128>, mg, dim3(256), 0, st, p, (int)Hkv, p.G);
        AGENTSAM_LAUNCH_CHECK();
    }
    return AGENTSAM_OK;
}
