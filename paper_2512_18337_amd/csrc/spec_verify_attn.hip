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

#include <algorithm>
#include <atomic>

#include "common.h"

// Workspace of spec_verify_attn_static: one copy per GPU the library runs on, held until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress; the kernels get the device
// address that call returns.
static __device__ __align__(256) unsigned char scratch[AGENTSAM_STATIC_WORKSPACE_BYTES];

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;          // finite stand-in for -inf in running maxima
constexpr float kPadRef = 1.0e30f;           // softmax reference of a row slot that holds no row
constexpr int kTile = 32;                    // KV positions per wavefront step
constexpr int kWaves = 4;
constexpr int kRowsPerGroup = 48;            // packed rows one wavefront can hold (3 MFMA row tiles of 16)
constexpr int kF32Chunk = 256;               // KV positions per workgroup of the fp32 kernel
constexpr int kF32MaxR = 32;

struct AttnParams {
    const void *q, *kc, *vc;
    const int32_t *bt, *seq;
    void *out;
    float *ws;
    int B, R, Hq, Hkv, G, D, P, max_pages;
    int log2P;               // log2(P) when P is a power of two, else -1
    int64_t num_pages;
    float scale_log2;        // scale * log2(e)
    int chunk;               // KV positions per workgroup
    int nchunks_max;         // grid extent over chunks
    int rows;                // G*R packed rows per kv head
    int rows_pad;            // rows per workspace record
    int out_bf16;
    int balanced;            // 1: balanced partition of the whole batch over the grid, 0: chunk grid
    int32_t *plan;           // balanced only: exclusive prefix sums of the sessions' tile counts, [B+1]
    float *wsr;              // workspace records (after the plan, if any)
    // shared-prefix ("cascade") run: the pages every session has in common are processed once per GROUP
    // of gs sessions (phase 1, wide kernel over gs*rows1 packed rows), the rest per session (phase 0)
    int cascade;             // 1: this launch is part of a cascade run
    int phase;               // 1: prefix phase of a cascade run
    int gs, ngroups;         // sessions per group, number of groups
    int rows1;               // packed rows of ONE session (G*R); == rows except in the prefix phase
    int rows_pad_p;          // rows per prefix record
    int nslots;              // workgroups of the balanced (suffix) launch
    const int32_t *lcp;      // [B] pages each session has in common with session 0 (written by attn_lcp_kernel)
    float *wsp;              // prefix records
};

// A session of S positions is cut into ceil(S / max_chunk) chunks of EQUAL size (rounded up to 128
// positions), so a ragged batch has no tiny trailing workgroups: every workgroup streams between
// half a maximum chunk and a full one.
__device__ __forceinline__ void chunk_geometry(int S, int max_chunk, int &nchunks, int &chunk_len) {
    nchunks = (S + max_chunk - 1) / max_chunk;
    chunk_len = nchunks > 0 ? (((S + nchunks - 1) / nchunks + 127) & ~127) : max_chunk;
}

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

// A row that sees no KV position (seq_lens[b] - R + i < 0, in particular every row of an empty
// session) has no softmax; its output is defined as zeros.
__device__ __forceinline__ float inv_or_zero(float l) { return l > 0.f ? 1.0f / l : 0.f; }

// zeros for every row of the query heads [h0, h0+nh) of session b (called by a whole workgroup)
__device__ __forceinline__ void zero_session_heads(const void *out_, int out_bf16, int b, int R, int Hq, int D, int h0, int nh) {
    void *out = const_cast<void *>(out_);
    const int per_row = nh * D / 4;                          // the heads of one query row are contiguous
    for (int idx = threadIdx.x; idx < R * per_row; idx += blockDim.x) {
        const int i = idx / per_row, c = idx % per_row;
        store_out(out, (((int64_t)b * R + i) * Hq + h0) * D + c * 4, float4{0.f, 0.f, 0.f, 0.f}, out_bf16);
    }
}

// ------------------------------------------------------------------------------------------
// bf16 MFMA kernels
// ------------------------------------------------------------------------------------------
template <int D>
struct Bf16Cfg {
    static constexpr int kKStr = D * 2 + 16;                 // LDS row strides in bytes (padded against
    static constexpr int kVStr = D * 2 + 32;                 // bank conflicts of the two read patterns)
    static constexpr int kTileBytes = kTile * (kKStr + kVStr);
    static constexpr int kOStr = D + 4;                      // floats
    static constexpr int kLoads = D / 16;                    // 16-byte loads per lane per tile, for K and for V
    static constexpr int kLanesPerRow = D / 8;
    static constexpr int kRowsPerLoad = 64 / kLanesPerRow;
};

__device__ __forceinline__ void wave_lds_fence() {
    // LDS operations of one wavefront execute in order; this only stops the compiler from moving
    // LDS accesses of different lanes across the point where a tile changes hands.
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ void wait_vmcnt0() {
    // s_waitcnt with only the vmcnt field active (gfx9 encoding: vmcnt[3:0] | expcnt<<4 | lgkmcnt<<8 | vmcnt[5:4]<<14)
    __builtin_amdgcn_s_waitcnt(0x0f70);
}

__device__ __forceinline__ uint4 ld_stream(const void *ptr) {
    // K/V are read exactly once per launch: keep them from displacing reusable lines
    const u32x4 v = __builtin_nontemporal_load((const u32x4 *)ptr);
    return uint4{v[0], v[1], v[2], v[3]};
}

// Returns x, but opaque to the optimiser: index arithmetic derived from the result is not hoisted out
// of an enclosing loop (where it would sit in registers across the whole tile loop).
__device__ __forceinline__ int opaque(int x) {
    asm volatile("" : "+v"(x));
    return x;
}

// Per-wavefront state: the packed query rows [row0, row_end) of one kv head, their running softmax
// statistics and the transposed output accumulators.
template <int D, int MT>
struct WaveState {
    bf16x8 qf[MT][D / 32];       // B operand of S^T = K.Q^T: column n = packed row, 8 consecutive d per lane
    int irow[MT];                // query row (0..R-1) of this lane's column, per row tile
    f32x4 oacc[D / 16][MT];      // O^T[d = 16*dt + 4g + r][row = 16*rt + n]
    float m_run[MT];             // reference maximum (base-2 domain), identical in the 4 lanes of a column
    float l_part[MT];            // this lane's share of the row sum
};

template <int D, int MT>
__device__ __forceinline__ void init_state(WaveState<D, MT> &w, const AttnParams &p, int b, int kvh,
                                           int row0, int row_end, int n_in, int g_in) {
    const int n = opaque(n_in), g = opaque(g_in);            // per-segment work: keep its index arithmetic here
    const __hip_bfloat16 *qg = (const __hip_bfloat16 *)p.q;
    const int R = p.R;
#pragma unroll
    for (int rt = 0; rt < MT; ++rt) {
        const int pr = row0 + rt * 16 + n;
        const bool live = pr < row_end;
        const int so = live ? pr / p.rows1 : 0;              // session within the group (0 outside the prefix phase)
        const int r1 = live ? pr - so * p.rows1 : 0;
        const int hh = live ? r1 / R : 0;
        const int i = live ? r1 % R : R - 1;
        w.irow[rt] = i;
        const __hip_bfloat16 *src = qg + (((int64_t)(b + so) * R + i) * p.Hq + (int64_t)kvh * p.G + hh) * D;
#pragma unroll
        for (int ks = 0; ks < D / 32; ++ks) {
            s16x8 raw = {0, 0, 0, 0, 0, 0, 0, 0};
            if (live) raw = *(const s16x8 *)(src + ks * 32 + g * 8);
            w.qf[rt][ks] = __builtin_bit_cast(bf16x8, raw);
        }
        // A row slot beyond the live rows gets a reference no score comes near: its weights are exact zeros, so the
        // second contraction multiplies zeros for it instead of accumulating sums of V that nobody reads.
        w.m_run[rt] = live ? kNegBig : kPadRef;
        w.l_part[rt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) w.oacc[dt][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
}

// max over the 4 lanes {n, n+16, n+32, n+48} that hold one packed row, result in all 4
__device__ __forceinline__ float row_max4(float x) {
    // v_permlane32_swap exchanges the upper half of the first operand with the lower half of the
    // second; with both operands equal the two results are x[l%32] and x[32 + l%32] in every lane.
    // v_permlane16_swap does the same for odd/even rows of 16 lanes.
    const unsigned xi = __float_as_uint(x);
    const u32x2 a = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
    const float m = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    const unsigned mi = __float_as_uint(m);
    const u32x2 c = __builtin_amdgcn_permlane16_swap(mi, mi, false, false);
    return fmaxf(__uint_as_float(c[0]), __uint_as_float(c[1]));
}

// S^T = K . Q^T for one 32-position tile: two 16-position tiles x MT row tiles
template <int D, int MT>
__device__ __forceinline__ void s_mfma(const WaveState<D, MT> &w, const char *Ks, f32x4 (&sacc)[2][MT], int n, int g) {
    using C = Bf16Cfg<D>;
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
                sacc[pt][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[pt], w.qf[rt][ks], sacc[pt][rt], 0, 0, 0);
    }
}

// Online softmax, part 1: bring the scores into the base-2 domain (masked ones to -inf) and find the
// row maxima.  Returns whether some row's maximum exceeds its reference by more than kSlack.
// The reference only moves in that case: any reference gives the same result after normalisation,
// weights stay below 2^kSlack, and the accumulators are rescaled a handful of times per wavefront
// instead of once per tile.
template <int D, int MT, bool MASK>
__device__ __forceinline__ bool softmax_max(const WaveState<D, MT> &w, f32x4 (&sacc)[2][MT], float (&mx)[MT],
                                            int pos0, int S, int R, float c, int g) {
    constexpr float kSlack = 8.0f;
    bool move = false;
#pragma unroll
    for (int rt = 0; rt < MT; ++rt) {
        if (MASK) {
            const int limit = S - R + w.irow[rt];            // last visible position of this row
#pragma unroll
            for (int pt = 0; pt < 2; ++pt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int pos = pos0 + pt * 16 + 4 * g + r;
                    sacc[pt][rt][r] = (pos <= limit) ? sacc[pt][rt][r] * c : -INFINITY;
                }
        }
        float m = fmaxf(fmaxf(sacc[0][rt][0], sacc[0][rt][1]), fmaxf(sacc[0][rt][2], sacc[0][rt][3]));
        m = fmaxf(m, fmaxf(fmaxf(sacc[1][rt][0], sacc[1][rt][1]), fmaxf(sacc[1][rt][2], sacc[1][rt][3])));
        m = row_max4(m);
        mx[rt] = MASK ? m : m * c;                           // c > 0
        move = move || (mx[rt] > w.m_run[rt] + kSlack);
    }
    return __builtin_amdgcn_ballot_w64(move) != 0;           // uniform over the wavefront, rarely true
}

// Move the reference maxima to max(old, mx) and rescale sums and accumulators accordingly.
template <int D, int MT>
__device__ __forceinline__ void rescale(WaveState<D, MT> &w, const float (&mx)[MT]) {
#pragma unroll
    for (int rt = 0; rt < MT; ++rt) {
        const float m_new = fmaxf(w.m_run[rt], mx[rt]);
        const float alpha = __builtin_amdgcn_exp2f(w.m_run[rt] - m_new);
        w.m_run[rt] = m_new;
        w.l_part[rt] *= alpha;
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) w.oacc[dt][rt] *= alpha;
    }
}

// Online softmax, part 2: weights 2^(s*c - m), rounded to bf16 for the second contraction (k-slot
// 8g+j <-> position j<4 ? 4g+j : 16+4g+j-4), and their row sums.  The sums are taken over the ROUNDED
// weights (packed dot product with ones, one instruction per two weights): numerator and denominator of
// the output then use the same weights, so a row dominated by a few keys is not off by the rounding
// error of its largest weight.
template <int D, int MT, bool MASK>
__device__ __forceinline__ void softmax_exp(WaveState<D, MT> &w, const f32x4 (&sacc)[2][MT], float c,
                                            bf16x8 (&pf)[MT]) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef short s16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 ones = __builtin_bit_cast(bf16x2, s16x2{0x3f80, 0x3f80});
#pragma unroll
    for (int rt = 0; rt < MT; ++rt) {
        const float mref = w.m_run[rt];
        float psum = w.l_part[rt];
        u32x4 pw;                                            // the 8 weights, packed two per register
#pragma unroll
        for (int pt = 0; pt < 2; ++pt)
#pragma unroll
            for (int r = 0; r < 4; r += 2) {
                const float e0 = MASK ? __builtin_amdgcn_exp2f(sacc[pt][rt][r] - mref)   // -inf -> 0
                                      : __builtin_amdgcn_exp2f(fmaf(sacc[pt][rt][r], c, -mref));
                const float e1 = MASK ? __builtin_amdgcn_exp2f(sacc[pt][rt][r + 1] - mref)
                                      : __builtin_amdgcn_exp2f(fmaf(sacc[pt][rt][r + 1], c, -mref));
                const bf16x2 pr = {(__bf16)e0, (__bf16)e1};
                psum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, psum, false);
                pw[pt * 2 + r / 2] = __builtin_bit_cast(unsigned, pr);   // the same register feeds the MFMA
            }
        w.l_part[rt] = psum;
        pf[rt] = __builtin_bit_cast(bf16x8, pw);
    }
}

// O^T += V^T . P^T for one tile
template <int D, int MT>
__device__ __forceinline__ void pv_mfma(WaveState<D, MT> &w, const char *Vs, const bf16x8 (&pf)[MT], int n, int g) {
    using C = Bf16Cfg<D>;
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) {
        bf16x8 vf;
        {
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
        }
#pragma unroll
        for (int rt = 0; rt < MT; ++rt)
            w.oacc[dt][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[rt], w.oacc[dt][rt], 0, 0, 0);
    }
}

// One 32-position tile (K at Ks, V at Vs in LDS) against the wavefront's rows, start to finish.
template <int D, int MT>
__device__ __forceinline__ void compute_tile(WaveState<D, MT> &w, const char *Ks, const char *Vs, int pos0,
                                             int S, int R, float c /* scale*log2e */, int n, int g) {
    f32x4 sacc[2][MT];
    bf16x8 pf[MT];
    s_mfma<D, MT>(w, Ks, sacc, n, g);
    float mx[MT];
    const bool mask = pos0 + kTile > S - R;                  // tile touches the new rows or the ragged end
    const bool move = mask ? softmax_max<D, MT, true>(w, sacc, mx, pos0, S, R, c, g)
                           : softmax_max<D, MT, false>(w, sacc, mx, pos0, S, R, c, g);
    if (move) rescale<D, MT>(w, mx);
    if (mask) softmax_exp<D, MT, true>(w, sacc, c, pf);
    else softmax_exp<D, MT, false>(w, sacc, c, pf);
    pv_mfma<D, MT>(w, Vs, pf, n, g);
}

// ------------------------------------------------------------------------------------------
// Work distribution.  A (session, kv head) pair is a stream of ceil(S/32) tiles.  Two schedules:
//
//   chunk grid   every stream is cut into equal chunks of at most p.chunk positions; workgroup
//                (chunk, session, kv head), kv head fastest and chunk slowest.  Streams of different
//                sessions are cut at (nearly) the same positions and those pieces are dispatched
//                together, so sessions that share the pages of a prefix meet in the L2 / the memory-side
//                cache.  Used when there are fewer streams than about two per workgroup slot, where
//                every stream has to be split anyway.
//   balanced     the streams are laid end to end (session-major, kv head minor) and that sequence of
//                T tiles is cut into gridDim.x equal shares, one per workgroup, all resident at once.
//                A workgroup walks its share segment by segment; only its first and last segment can
//                be part of a stream (everything in between is a whole stream, written out directly),
//                so there are at most two partial records per workgroup and no tail of unevenly sized
//                workgroups, however ragged the batch.  seq_lens lives on the device, so every
//                workgroup derives its share itself: a block-wide scan of the tile counts.
// ------------------------------------------------------------------------------------------
constexpr int kMinShare = 4;                 // tiles; smaller problems leave workgroups idle

struct Segment {
    int b, kvh, S;           // session, kv head, clamped sequence length
    int t0, nt;              // tile range [t0, t0+nt) of the stream
    int64_t rec;             // workspace record for the partial result, -1: whole stream, write the output
    int rows;                // packed rows that are live in this segment (a short last group has fewer)
};

__device__ __forceinline__ int session_len(const AttnParams &p, int b) {
    return max(0, min(p.seq[b], p.max_pages * p.P));         // never index past the block table
}
__device__ __forceinline__ int tiles_of(int S) { return S > 0 ? (S + kTile - 1) / kTile : 0; }

// exclusive prefix of v over the 256 threads of the workgroup, and the total; `tmp` is 4 ints of LDS
__device__ __forceinline__ int block_scan_excl(int v, int *tmp, int &total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int u = __shfl_up(incl, off, 64);
        if (lane >= off) incl += u;
    }
    if (lane == 63) tmp[wave] = incl;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int ww = 0; ww < kWaves; ++ww) {
        const int x = tmp[ww];
        if (ww < wave) base += x;
        tot += x;
    }
    __syncthreads();                                         // tmp may be reused
    total = tot;
    return base + incl - v;
}

// minimum of v over the 256 threads of the workgroup; `tmp` is 4 ints of LDS
__device__ __forceinline__ int block_min(int v, int *tmp) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = min(v, __shfl_xor(v, off, 64));
    if (lane == 0) tmp[wave] = v;
    __syncthreads();
    int m = tmp[0];
#pragma unroll
    for (int ww = 1; ww < kWaves; ++ww) m = min(m, tmp[ww]);
    __syncthreads();
    return m;
}

// Tiles of the prefix all sessions share (cascade runs): whole pages that every session lists at the
// same place of its block table and that lie in front of every session's new rows.
__device__ __forceinline__ int shared_prefix_tiles(const AttnParams &p, int *tmp) {
    int m = 0x7fffffff;
    for (int bb = threadIdx.x; bb < p.B; bb += 256) m = min(m, p.lcp[bb]);
    const int pages = __builtin_amdgcn_readfirstlane(block_min(m, tmp));
    return pages * (p.P / kTile);
}

__device__ __forceinline__ int balanced_share(int T, int nslots) {
    const int s = (T + nslots - 1) / nslots;
    return s < kMinShare ? kMinShare : s;
}

// Calls body(Segment) for every segment of workgroup `wg` of `nwg`, in order.  `tmp`: 8 ints of LDS that
// the body does not touch.  Everything handed to the body is uniform over the workgroup (scalar registers).
template <class Body>
__device__ __forceinline__ void for_each_segment(const AttnParams &p, int *tmp, int wg, int nwg, Body body) {
    Segment sg;
    sg.rows = p.rows;
    int nt_b;                    // tiles of the current stream (chunk grid: end of my chunk)
    int remaining;               // tiles of my share still to do
    int64_t chunk_rec = -1;      // chunk grid: the one record
    int ptiles = 0;              // cascade: tiles of the shared prefix, which the streams below start after
    if (p.cascade) ptiles = shared_prefix_tiles(p, tmp);
    if (p.phase == 1) {
        // prefix phase: the streams are (group, kv head) pairs, all ptiles long, laid end to end (kv head minor)
        // and cut into nwg equal shares.  The group's sessions share these tiles, so their rows are packed side
        // by side and the block table of the group's first session serves all.
        const int T = p.ngroups * p.Hkv * ptiles;
        const int share = balanced_share(T, nwg);
        const int lo = wg * share;
        if (lo >= T) return;
        remaining = min(T, lo + share) - lo;
        const int s = lo / ptiles;
        sg.t0 = lo - s * ptiles;
        sg.kvh = s % p.Hkv;
        sg.b = (s / p.Hkv) * p.gs;
        sg.rows = min(p.gs, p.B - sg.b) * p.rows1;
        sg.S = ptiles * kTile + p.R;                         // every row sees the whole prefix: nothing is masked
        nt_b = ptiles;
    } else if (!p.balanced) {
        sg.kvh = wg % p.Hkv;
        sg.b = (wg / p.Hkv) % p.B;
        sg.S = session_len(p, sg.b);
        int nchunks_b, chunk_len;
        chunk_geometry(sg.S, p.chunk, nchunks_b, chunk_len);
        const int chunk = wg / (p.B * p.Hkv);
        if (sg.S <= 0 && chunk == 0) zero_session_heads(p.out, p.out_bf16, sg.b, p.R, p.Hq, p.D, sg.kvh * p.G, p.G);
        if (chunk >= nchunks_b) return;
        const int c0 = chunk * chunk_len, c1 = min(sg.S, c0 + chunk_len);
        sg.t0 = c0 / kTile;                                  // chunk_len is a multiple of 128
        remaining = (c1 - c0 + kTile - 1) / kTile;
        nt_b = sg.t0 + remaining;
        if (nchunks_b > 1) chunk_rec = ((int64_t)sg.b * p.Hkv + sg.kvh) * p.nchunks_max + chunk;
    } else {
        const int tid = threadIdx.x;
        // pass 1: T
        int sessions_tiles = 0;
        for (int base = 0; base < p.B; base += 256) {
            const int bb = base + tid;
            int tot;
            block_scan_excl(bb < p.B ? max(0, tiles_of(session_len(p, bb)) - ptiles) : 0, tmp, tot);
            sessions_tiles += tot;
        }
        const int T = __builtin_amdgcn_readfirstlane(sessions_tiles) * p.Hkv;   // uniform: scalar registers
        const int share = balanced_share(T, nwg);
        const int lo = wg * share;
        if (wg != 0 && lo >= T) return;                      // workgroup 0 stays to write the plan
        // pass 2: the stream my share starts in; workgroup 0 also leaves the prefix sums for the merge
        int carry = 0;
        if (tid == 0) tmp[4] = -1;                           // ordered before the writes below by the scan's barriers
        for (int base = 0; base < p.B; base += 256) {
            const int bb = base + tid;
            const int nt = bb < p.B ? max(0, tiles_of(session_len(p, bb)) - ptiles) : 0;
            int tot;
            const int excl = carry + block_scan_excl(nt, tmp, tot);
            if (wg == 0 && bb < p.B) p.plan[bb] = excl;
            if (nt > 0 && excl * p.Hkv <= lo && lo < (excl + nt) * p.Hkv) { tmp[4] = bb; tmp[5] = excl; }
            carry += tot;
        }
        if (wg == 0 && tid == 0) p.plan[p.B] = carry;
        __syncthreads();
        if (lo >= T) return;
        sg.b = __builtin_amdgcn_readfirstlane(tmp[4]);
        if (sg.b < 0 || sg.b >= p.B) return;                 // cannot happen: some stream contains tile `lo`
        const int excl0 = __builtin_amdgcn_readfirstlane(tmp[5]);
        sg.S = __builtin_amdgcn_readfirstlane(session_len(p, sg.b));
        nt_b = max(0, tiles_of(sg.S) - ptiles);
        const int r = lo - excl0 * p.Hkv;
        sg.kvh = r / nt_b;
        sg.t0 = r % nt_b;
        remaining = min(T, lo + share) - lo;
    }
    bool first = true;
    while (remaining > 0) {                                  // (one round on the chunk grid)
        sg.nt = min(remaining, nt_b - sg.t0);
        const bool whole = sg.t0 == 0 && sg.nt == nt_b;
        if (p.phase == 1) {
            // one record per (workgroup, stream) pair that occurs.  Walking the shares in order, every new
            // segment moves on by one workgroup, by one stream, or by both, so wg + stream index is a
            // different number for every segment and stays below nwg + number of streams.
            sg.rec = (int64_t)wg + (sg.b / p.gs) * p.Hkv + sg.kvh;
            body(sg);
        } else {
            if (!p.balanced) sg.rec = chunk_rec;
            else if (p.cascade) sg.rec = (whole && ptiles == 0) ? -1 : (int64_t)wg + (int64_t)sg.b * p.Hkv + sg.kvh;   // (as in the prefix phase)
            else sg.rec = whole ? -1 : 2 * (int64_t)wg + (first ? 0 : 1);
            if (ptiles > 0) {                                // the stream's tiles come after the shared prefix
                Segment abs = sg;
                abs.t0 += ptiles;
                body(abs);
            } else {
                body(sg);
            }
        }
        remaining -= sg.nt;
        first = false;
        sg.t0 = 0;
        if (remaining > 0 && ++sg.kvh == p.Hkv) {
            sg.kvh = 0;
            if (p.phase == 1) {                              // next group
                sg.b += p.gs;
                if (sg.b >= p.B) return;                     // cannot happen: the shares end with the last group
                sg.rows = min(p.gs, p.B - sg.b) * p.rows1;
            } else {
                do {                                         // sessions without tiles own no part of the sequence
                    ++sg.b;
                    if (sg.b >= p.B) return;                 // cannot happen while seq_lens is unchanged
                    sg.S = __builtin_amdgcn_readfirstlane(session_len(p, sg.b));
                    nt_b = max(0, tiles_of(sg.S) - ptiles);
                } while (nt_b == 0);
            }
        }
    }
}

// A session's row of the block table, read through the constant address space: the table does not change
// during a launch, so a load with a uniform index is a scalar load, which neither takes vector registers
// nor counts among the vector loads in flight.
typedef const int32_t __attribute__((address_space(4))) *BlockTableRow;
__device__ __forceinline__ BlockTableRow block_table_row(const AttnParams &p, int b) {
    return (BlockTableRow)(uintptr_t)(p.bt + (int64_t)b * p.max_pages);
}

// Largest chunk of the chunk grid, in KV positions.
constexpr int kMaxChunk = 256 * kTile;
// Wide kernel: where this many tiles of a segment lie in the caches is held in LDS (4 KB; with the tile ring 68 KB
// per workgroup, two workgroups per compute unit).  A longer segment (more than 32768 positions of one stream in
// one workgroup's share) is taken in pieces of this size, the ring draining and refilling in between.  (Scalar loads of the block table at the point of the request, as
// the narrow kernel makes them one step ahead, were measured here too: 1 to 2 % slower, the request being on the
// critical path of a tile.)
constexpr int kPageIds = 1024;

// -------- narrow kernel: up to 48 packed rows; the 4 wavefronts take different tiles of the segment
template <int D, int MT>
__global__ __launch_bounds__(256) void attn_bf16_narrow_kernel(const AttnParams p) {
    using C = Bf16Cfg<D>;
    constexpr int kStage = kWaves * C::kTileBytes;
    constexpr int kMerge = kRowsPerGroup * C::kOStr * 4;
    __shared__ __align__(16) char smem[kStage > kMerge ? kStage : kMerge];
    __shared__ float red_m[kWaves * kRowsPerGroup];
    __shared__ float red_l[kWaves * kRowsPerGroup];
    __shared__ int sched_tmp[8];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;   // wave index lives in an SGPR
    const int n = lane & 15, g = lane >> 4;
    const int R = p.R;
    char *Ks = smem + wave * C::kTileBytes;
    char *Vs = Ks + kTile * C::kKStr;
    // tile loads: lane -> (row, 16-byte column); one instruction reads 1 KB contiguous
    const int ld_row = lane / C::kLanesPerRow, ld_col = lane % C::kLanesPerRow;

    for_each_segment(p, sched_tmp, (int)blockIdx.x, (int)gridDim.x, [&](const Segment &sg) __attribute__((always_inline)) {
        const int b = sg.b, kvh = sg.kvh, S = sg.S;
        WaveState<D, MT> w;
        init_state<D, MT>(w, p, b, kvh, 0, p.rows, n, g);

        // My tiles of the segment: i-th one is tile t_first + 4*i of the stream.  Its page id comes from the
        // block table with a scalar load (uniform address, read-only for the whole launch), fetched one step
        // before the tile is requested, so the tile loop neither waits for it nor has a vector load of its
        // own between the streaming loads whose completion it counts, and a segment of any length runs
        // as one uninterrupted pipeline.
        const BlockTableRow bt_row = block_table_row(p, b);
        const int t_first = sg.t0 + wave;
        const int n_my = wave < sg.nt ? (sg.nt - wave + kWaves - 1) / kWaves : 0;   // tiles of this wavefront
        auto page_of = [&](int i) {                              // uniform; -1 past my last tile
            if (i >= n_my) return -1;
            const int pos0 = (t_first + kWaves * i) * kTile;
            return (int)bt_row[p.log2P >= 0 ? (pos0 >> p.log2P) : (pos0 / p.P)];
        };
        auto usable = [&](int page) { return page >= 0 && (int64_t)page < p.num_pages; };

        // Two tiles are kept in flight in registers while a third is being computed from LDS.  The
        // loads are issued unconditionally (past the wavefront's last tile every lane re-reads the first
        // bytes of q, one hot cache line; an unusable page id reads page 0) and what must not be seen
        // is zeroed when the tile is staged:
        // with a fixed number of loads per step the compiler can wait for exactly the older of the two
        // tiles in flight instead of for everything outstanding.
        uint4 kreg[2][C::kLoads], vreg[2][C::kLoads];
        auto issue_loads = [&](int i, int page, uint4 (&kr)[C::kLoads], uint4 (&vr)[C::kLoads]) {
            const bool live = i < n_my;                          // uniform
            const int pos0 = (t_first + kWaves * i) * kTile;
            const int slot = p.log2P >= 0 ? (pos0 & (p.P - 1)) : (pos0 % p.P);
            const int64_t base = (((int64_t)(usable(page) ? page : 0) * p.Hkv + kvh) * p.P + slot) * D;
            const __hip_bfloat16 *kb = live ? (const __hip_bfloat16 *)p.kc + base : (const __hip_bfloat16 *)p.q;
            const __hip_bfloat16 *vb = live ? (const __hip_bfloat16 *)p.vc + base : (const __hip_bfloat16 *)p.q;
            const int lane_off = live ? ld_row * D + ld_col * 8 : 0;
            const int step = live ? C::kRowsPerLoad * D : 0;
#pragma unroll
            for (int j = 0; j < C::kLoads; ++j) {
                kr[j] = ld_stream(kb + lane_off + j * step);
                vr[j] = ld_stream(vb + lane_off + j * step);
            }
        };
        auto stage = [&](int i, int page, const uint4 (&kr)[C::kLoads], const uint4 (&vr)[C::kLoads]) {
            const int pos0 = (t_first + kWaves * i) * kTile;
            const bool page_ok = usable(page);
            if (page_ok && pos0 + kTile <= S) {                  // the usual case: a full tile
#pragma unroll
                for (int j = 0; j < C::kLoads; ++j) {
                    const int row = j * C::kRowsPerLoad + ld_row;
                    *(uint4 *)(Ks + row * C::kKStr + ld_col * 16) = kr[j];
                    *(uint4 *)(Vs + row * C::kVStr + ld_col * 16) = vr[j];
                }
            } else {                                             // rows past the end, or a page of zeros
#pragma unroll
                for (int j = 0; j < C::kLoads; ++j) {
                    const int row = j * C::kRowsPerLoad + ld_row;
                    const bool ok = page_ok && pos0 + row < S;
                    *(uint4 *)(Ks + row * C::kKStr + ld_col * 16) = ok ? kr[j] : uint4{0u, 0u, 0u, 0u};
                    *(uint4 *)(Vs + row * C::kVStr + ld_col * 16) = ok ? vr[j] : uint4{0u, 0u, 0u, 0u};
                }
            }
        };

        // Stage tile i_st out of (kr, vr) and request tile i_rq into the same registers.  For a full tile each
        // register is written to LDS and loaded again at once, so the first requests of the new tile go out
        // before the staging of the old one is over.
        auto stage_and_issue = [&](int i_st, int page_st, int i_rq, int page_rq, uint4 (&kr)[C::kLoads],
                                   uint4 (&vr)[C::kLoads]) {
            const int pos_st = (t_first + kWaves * i_st) * kTile;
            if (!(usable(page_st) && pos_st + kTile <= S)) {
                stage(i_st, page_st, kr, vr);
                issue_loads(i_rq, page_rq, kr, vr);
                return;
            }
            const bool live = i_rq < n_my;                       // uniform
            const int pos0 = (t_first + kWaves * i_rq) * kTile;
            const int slot = p.log2P >= 0 ? (pos0 & (p.P - 1)) : (pos0 % p.P);
            const int64_t base = (((int64_t)(usable(page_rq) ? page_rq : 0) * p.Hkv + kvh) * p.P + slot) * D;
            const __hip_bfloat16 *kb = live ? (const __hip_bfloat16 *)p.kc + base : (const __hip_bfloat16 *)p.q;
            const __hip_bfloat16 *vb = live ? (const __hip_bfloat16 *)p.vc + base : (const __hip_bfloat16 *)p.q;
            const int lane_off = live ? ld_row * D + ld_col * 8 : 0;
            const int step = live ? C::kRowsPerLoad * D : 0;
#pragma unroll
            for (int j = 0; j < C::kLoads; ++j) {
                const int row = j * C::kRowsPerLoad + ld_row;
                *(uint4 *)(Ks + row * C::kKStr + ld_col * 16) = kr[j];
                *(uint4 *)(Vs + row * C::kVStr + ld_col * 16) = vr[j];
                kr[j] = ld_stream(kb + lane_off + j * step);
                vr[j] = ld_stream(vb + lane_off + j * step);
            }
        };

        if (n_my > 0) {
            int pg0 = page_of(0), pg1 = page_of(1), pg_next = page_of(2);
            // Nothing else may be outstanding when the tile pipeline starts: with only its own loads in
            // flight, in a known order, the compiler's waits inside the loop count exactly; a pending load
            // of the query fragments or a store of the previous segment would make every wait at the top of
            // the loop a wait for everything.
            wait_vmcnt0();
            issue_loads(0, pg0, kreg[0], vreg[0]);
            issue_loads(1, pg1, kreg[1], vreg[1]);
            // Two tiles per round, so that the two register sets keep their roles; an odd last tile follows
            // the loop.  The loop has one exit, at its end: an exit between the two halves would give the
            // first half a path on which its own loads are the newest in flight, and the waits in front of
            // its staging would then have to cover the other tile's loads as well.
            int i = 0;
            for (; i + 1 < n_my; i += 2) {
                stage_and_issue(i, pg0, i + 2, pg_next, kreg[0], vreg[0]);
                pg0 = pg_next;
                wave_lds_fence();
                pg_next = page_of(i + 3);
                compute_tile<D, MT>(w, Ks, Vs, (t_first + kWaves * i) * kTile, S, R, p.scale_log2, n, g);
                wave_lds_fence();
                stage_and_issue(i + 1, pg1, i + 3, pg_next, kreg[1], vreg[1]);
                pg1 = pg_next;
                wave_lds_fence();
                pg_next = page_of(i + 4);
                compute_tile<D, MT>(w, Ks, Vs, (t_first + kWaves * (i + 1)) * kTile, S, R, p.scale_log2, n, g);
                wave_lds_fence();
            }
            if (i < n_my) {
                stage(i, pg0, kreg[0], vreg[0]);
                wave_lds_fence();
                compute_tile<D, MT>(w, Ks, Vs, (t_first + kWaves * i) * kTile, S, R, p.scale_log2, n, g);
                wave_lds_fence();
            }
        }

        // ---- merge the 4 wavefronts through LDS
        const int n_e = opaque(n), g_e = opaque(g), tid_e = opaque(tid);   // not hoisted out of the segment loop
        float l_tot[MT];
#pragma unroll
        for (int rt = 0; rt < MT; ++rt) {
            float l = w.l_part[rt];
            l += __shfl_xor(l, 16, 64);
            l += __shfl_xor(l, 32, 64);
            l_tot[rt] = l;
        }
        __syncthreads();                                     // staging LDS is free from here on
        if (g_e == 0) {
#pragma unroll
            for (int rt = 0; rt < MT; ++rt) {
                red_m[wave * kRowsPerGroup + rt * 16 + n_e] = w.m_run[rt];
                red_l[wave * kRowsPerGroup + rt * 16 + n_e] = l_tot[rt];
            }
        }
        __syncthreads();
        float my_scale[MT], M_all[MT], L_all[MT];
#pragma unroll
        for (int rt = 0; rt < MT; ++rt) {
            const int row = rt * 16 + n_e;
            float M = red_m[row];
#pragma unroll
            for (int ww = 1; ww < kWaves; ++ww) M = fmaxf(M, red_m[ww * kRowsPerGroup + row]);
            float L = 0.f;
#pragma unroll
            for (int ww = 0; ww < kWaves; ++ww)
                L += red_l[ww * kRowsPerGroup + row] * __builtin_amdgcn_exp2f(red_m[ww * kRowsPerGroup + row] - M);
            M_all[rt] = M;
            L_all[rt] = L;
            my_scale[rt] = __builtin_amdgcn_exp2f(w.m_run[rt] - M);
        }
        float *Osum = (float *)smem;
        for (int ww = 0; ww < kWaves; ++ww) {
            if (wave == ww) {
#pragma unroll
                for (int rt = 0; rt < MT; ++rt)
#pragma unroll
                    for (int dt = 0; dt < D / 16; ++dt) {
                        float4 *dst = (float4 *)(Osum + (rt * 16 + n_e) * C::kOStr + dt * 16 + 4 * g_e);
                        const f32x4 a = w.oacc[dt][rt] * my_scale[rt];
                        float4 v{a[0], a[1], a[2], a[3]};
                        if (ww > 0) { const float4 o = *dst; v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w; }
                        *dst = v;
                    }
            }
            __syncthreads();
        }
        // every wavefront computed the same merged maximum and sum; the per-wavefront entries were last
        // read before the barriers above, so wavefront 0 may now overwrite its own with the merged values
        if (wave == 0 && g_e == 0) {
#pragma unroll
            for (int rt = 0; rt < MT; ++rt) { red_m[rt * 16 + n_e] = M_all[rt]; red_l[rt * 16 + n_e] = L_all[rt]; }
        }
        __syncthreads();

        const int rows_here = p.rows;
        if (sg.rec < 0) {
            for (int idx = tid_e; idx < rows_here * (D / 4); idx += 256) {
                const int row = idx / (D / 4), c4 = idx % (D / 4);
                const int hh = row / R, i = row % R;
                const float inv = inv_or_zero(red_l[row]);
                float4 v = *(const float4 *)(Osum + row * C::kOStr + c4 * 4);
                v.x *= inv; v.y *= inv; v.z *= inv; v.w *= inv;
                const int64_t o = (((int64_t)b * R + i) * p.Hq + (int64_t)kvh * p.G + hh) * D + c4 * 4;
                store_out(p.out, o, v, p.out_bf16);
            }
        } else {
            float *wo = p.wsr + sg.rec * ws_record_floats(p.rows_pad, D);
            float *wm = wo + (int64_t)p.rows_pad * D;
            float *wl = wm + p.rows_pad;
            for (int idx = tid_e; idx < rows_here * (D / 4); idx += 256) {
                const int row = idx / (D / 4), c4 = idx % (D / 4);
                *(float4 *)(wo + (int64_t)row * D + c4 * 4) = *(const float4 *)(Osum + row * C::kOStr + c4 * 4);
            }
            if (tid_e < rows_here) { wm[tid_e] = red_m[tid_e]; wl[tid_e] = red_l[tid_e]; }
        }
        __syncthreads();                                     // the next segment stages into the same LDS
    });
}

// -------- wide kernel: 49..192 packed rows; the 4 wavefronts take different rows of the SAME tile.
//
// With this many rows per K/V byte the MFMA and softmax arithmetic are no longer negligible next to
// the memory stream, and there are no registers to spare for staging, so:
//   - tiles go from global memory straight into a ring of NS LDS slots (global_load_lds_dwordx4:
//     lane i's 16 bytes land at slot base + 16*i).  The wavefronts take turns: tile t is fetched
//     whole by wavefront t % 4, so the address arithmetic of a tile is paid once, not four times,
//     and a wavefront only ever waits for the one tile it issued (s_waitcnt vmcnt(0));
//   - rows are stored unpadded (256 B for D=128), so the 16-byte chunks of a row are XOR-swizzled
//     with the row index on the way in (the lane picks which global chunk it fetches) to keep the
//     column-wise fragment reads off a single bank;
//   - the softmax reference of a row is FIXED at the maximum of the first tile in which the row sees
//     anything, so the steady-state tile is branch-free: weights 2^(s*c - ref), no running maximum,
//     no rescaling of the accumulators (any reference gives the same result after normalisation).
//     Should a later score exceed the reference by so much that a weight overflows - the sums then
//     turn non-finite or absurdly large - the chunk is redone: one pass that only raises the
//     references to the exact row maxima, then a final pass;
//   - registers stay under 256 so that two workgroups share a compute unit and one's wavefront
//     fills the other's stalls; one workgroup barrier per tile publishes the tile.
template <int D>
struct WideCfg {
    static constexpr int kRowBytes = D * 2;
    static constexpr int kKT = kTile * kRowBytes;            // bytes of the K (or V) part of a tile
    static constexpr int kSlot = 2 * kKT;
    static constexpr int kCPR = D / 8;                       // 16-byte chunks per row
    static constexpr int kRPI = 64 / kCPR;                   // rows per 1 KB load instruction
    static constexpr int kPieces = kTile / kRPI;             // 1 KB load instructions per K (or V) tile
    static constexpr int kG = kCPR > kRPI ? kCPR / kRPI : 1; // the swizzle pattern of a piece repeats every kG pieces
};

// 16 bytes per lane from global memory straight into LDS: lane i's data lands at lds_base + 16*i.
// Written as inline assembly on purpose: the compiler then neither reorders it (memory clobber) nor
// adds its own conservative "wait for every outstanding LDS-DMA" in front of later LDS reads;
// completion is awaited explicitly with s_waitcnt vmcnt(0) by the issuing wavefront.  An unknown VMEM
// instruction can only make the compiler's own vmcnt waits stricter, never weaker.
__device__ __forceinline__ void lds_dma16(const void *gbase /* uniform */, unsigned voff, unsigned lds_addr /* uniform */) {
    const unsigned m = __builtin_amdgcn_readfirstlane(lds_addr);
    unsigned saved;
    asm volatile(
        "s_mov_b32 %0, m0\n\t"
        "s_mov_b32 m0, %1\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %2, %3\n\t"
        "s_mov_b32 m0, %0"
        : "=&s"(saved)
        : "s"(m), "v"(voff), "s"(gbase)
        : "memory");
}

// Tell the compiler a pointer is the same in every lane (keeps it in a scalar register pair).
__device__ __forceinline__ const void *uniform_ptr(const void *ptr) {
    const uint64_t v = (uint64_t)ptr;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const void *)(((uint64_t)hi << 32) | lo);
}

// A whole tile (all 1 KB pieces of K, then of V at +kKT) in one block.  The instruction's immediate
// offset is added to the global AND to the LDS address, so four consecutive pieces share one M0
// value and one base register pair: M0 is written once per 4 KB, not once per piece.  goffp[i] is
// the lane's byte offset inside piece i of a group, without the piece's own i*1024 (the swizzle
// repeats every kG pieces, so kG offsets serve all pieces).
#define AGENTSAM_DMA_GROUP(MOFF, SB, G0, G1, G2, G3)                 \
    "s_add_u32 m0, %1, " MOFF "\n\ts_nop 0\n\t"                     \
    "global_load_lds_dwordx4 " G0 ", " SB " nt\n\t"                  \
    "global_load_lds_dwordx4 " G1 ", " SB " offset:1024 nt\n\t"      \
    "global_load_lds_dwordx4 " G2 ", " SB " offset:2048 nt\n\t"      \
    "global_load_lds_dwordx4 " G3 ", " SB " offset:3072 nt\n\t"
template <int D>
__device__ __forceinline__ void lds_dma_tile(const char *kb, const char *vb, const unsigned (&goffp)[WideCfg<D>::kG],
                                             unsigned slot_addr /* uniform LDS byte address */) {
    const unsigned m = __builtin_amdgcn_readfirstlane(slot_addr);
    unsigned saved;
    if constexpr (D == 128) {
        static_assert(WideCfg<D>::kPieces == 8 && WideCfg<D>::kG == 4, "two groups of four pieces");
        const char *kb1 = kb + 4096, *vb1 = vb + 4096;
        asm volatile("s_mov_b32 %0, m0\n\t"
                     AGENTSAM_DMA_GROUP("0", "%2", "%7", "%8", "%9", "%10")
                     AGENTSAM_DMA_GROUP("4096", "%4", "%7", "%8", "%9", "%10")
                     AGENTSAM_DMA_GROUP("%c6", "%3", "%7", "%8", "%9", "%10")
                     AGENTSAM_DMA_GROUP("%c6+4096", "%5", "%7", "%8", "%9", "%10")
                     "s_mov_b32 m0, %0"
                     : "=&s"(saved)
                     : "s"(m), "s"(kb), "s"(vb), "s"(kb1), "s"(vb1), "n"(WideCfg<D>::kKT), "v"(goffp[0]), "v"(goffp[1]),
                       "v"(goffp[2]), "v"(goffp[3])
                     : "memory", "scc");
    } else {
        static_assert(WideCfg<D>::kPieces == 4 && WideCfg<D>::kG == 1, "one group of four pieces");
        asm volatile("s_mov_b32 %0, m0\n\t"
                     AGENTSAM_DMA_GROUP("0", "%2", "%5", "%5", "%5", "%5")
                     AGENTSAM_DMA_GROUP("%c4", "%3", "%5", "%5", "%5", "%5")
                     "s_mov_b32 m0, %0"
                     : "=&s"(saved)
                     : "s"(m), "s"(kb), "s"(vb), "n"(WideCfg<D>::kKT), "v"(goffp[0])
                     : "memory", "scc");
    }
}
#undef AGENTSAM_DMA_GROUP

template <int D, int MT, int NS, bool XT>
__device__ __forceinline__ void wide_body(const AttnParams &p, char *smem, int *page_lds, int *sched_tmp, int wg, int nwg) {
    using W = WideCfg<D>;
    // (opaque: a kernel that runs two bodies one after the other computes each body's lane constants when
    // that body starts, instead of keeping both sets in registers across both)
    const int tid = opaque((int)threadIdx.x);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;   // wave index lives in an SGPR
    const int n = lane & 15, g = lane >> 4;
    const int R = p.R;
    const float c = p.scale_log2;

    // Row assignment.  Plain: rows split evenly, ceil(rows/4) per wavefront.  XT ("extra tile"): every
    // wavefront owns 16*MT rows outright and the remaining <= 16 rows form one more row tile that is
    // processed by wavefront t % 4 for tile t, so its work is spread evenly (136 rows = 4 x 32 + 8 cost
    // 2.25 row tiles per wavefront instead of 3); the four partial results of those rows are merged
    // at the end.
    const int rpw = XT ? 16 * MT : (p.rows + kWaves - 1) / kWaves;
    const int row0 = wave * rpw;
    constexpr int kXRow0 = kWaves * 16 * MT;                 // first extra row (XT only)

    // ---- per-lane constants of the tile loop (computed once; the loop only adds uniform bases)
    // piece j of a tile (1 KB = kRPI rows): my 16 bytes are row j*kRPI + lrow, and I fetch the global
    // chunk that belongs in my LDS chunk under the XOR swizzle
    const int lrow = lane / W::kCPR, lslot = lane % W::kCPR;
    unsigned goffp[W::kG];                                   // byte offset inside piece i (mod kG), minus the piece's i*1024
#pragma unroll
    for (int i = 0; i < W::kG; ++i)
        goffp[i] = (unsigned)(lrow * W::kRowBytes + (lslot ^ ((i * W::kRPI + lrow) & (W::kCPR - 1))) * 16);
    // fragment reads: K rows n and n+16 (the swizzle only sees row & 15), V rows 4g+jq and +16.
    // Under the XOR swizzle the offset for k-step ks is koff0 ^ (ks << 6) and for d-tile dt it is
    // voff0 ^ (dt << 5); since slot offsets are multiples of 16 KB the XOR can be applied after the
    // slot offset is added, so only two lane constants stay live.
    const int koff0 = n * W::kRowBytes + ((g ^ (n & (W::kCPR - 1))) * 16);
    int voff0;
    {
        const int bq = n & 3, jq = n >> 2, vrow = 4 * g + jq;    // transpose-read lane roles, see pv_mfma
        voff0 = W::kKT + vrow * W::kRowBytes + (((bq >> 1) ^ (vrow & (W::kCPR - 1))) * 16) + (bq & 1) * 8;
    }
    const unsigned smem_addr = (unsigned)(size_t)(__attribute__((address_space(3))) char *)smem;   // LDS byte address

    for_each_segment(p, sched_tmp, wg, nwg, [&](const Segment &sg) __attribute__((always_inline)) {
    const int b = sg.b, kvh = sg.kvh, S = sg.S;
    const int row_end = min(sg.rows, row0 + rpw);            // (a short last group of the prefix phase has fewer rows)
    WaveState<D, MT> w;
    init_state<D, MT>(w, p, b, kvh, row0, row_end, n, g);
    WaveState<D, 1> wx;
    if (XT) init_state<D, 1>(wx, p, b, kvh, kXRow0, sg.rows, n, g);

    // attempt: 0 optimistic (fixed references), 1 exact row maxima only, 2 final pass with those
    for (int attempt = 0;; ++attempt) {
      const bool raise_always = attempt == 1;
      // Where every tile of the segment lies in the caches sits in LDS (kPageIds tiles at a time: only a segment
      // longer than that drains and refills the ring in between); the wavefront that requests a tile reads the
      // place of the tile it will request next right after a request, so it is in a register when it is needed.
      for (int sub = 0; sub < sg.nt; sub += kPageIds) {
        const int c0 = (sg.t0 + sub) * kTile;
        const int ntiles = min(sg.nt - sub, kPageIds);
        {
            // what is kept per tile is its place in the caches, counted in tiles: ((page * Hkv + kv head) * P + slot) / 32,
            // or -1 for an unusable page id; the request then needs one shift and two additions
            const BlockTableRow bt_row = block_table_row(p, b);
            const int tiles_per_page = p.P / kTile;
            for (int i = tid; i < ntiles; i += 256) {
                const int pos = c0 + i * kTile;
                const int page = bt_row[p.log2P >= 0 ? (pos >> p.log2P) : (pos / p.P)];
                const int slot = p.log2P >= 0 ? (pos & (p.P - 1)) : (pos % p.P);
                const bool ok = page >= 0 && (int64_t)page < p.num_pages;
                page_lds[i] = ok ? (page * p.Hkv + kvh) * tiles_per_page + slot / kTile : -1;
            }
        }
        // The query fragments are needed at once; waiting for them here, explicitly, keeps the compiler from
        // guarding their first use inside the tile loop with a wait that would also drain the tile this
        // wavefront has just started to fetch.
        wait_vmcnt0();
        __syncthreads();                                     // the page ids are in place

    // fetch tile t into its ring slot (called by one wavefront)
    auto issue = [&](int t, int place, int slot_idx) {
        const int pos0 = c0 + t * kTile;
        const bool page_ok = place >= 0;
        const int64_t base = (int64_t)(page_ok ? place : 0) * (kTile * D * 2);
        const char *kb = (const char *)uniform_ptr((const char *)p.kc + base);
        const char *vb = (const char *)uniform_ptr((const char *)p.vc + base);
        const int slot_off = slot_idx * W::kSlot;
        const int rows_left = S - pos0;                      // rows >= rows_left lie past the sequence
        if (page_ok && rows_left >= kTile) {                 // the usual case: a full tile, all lanes load
            lds_dma_tile<D>(kb, vb, goffp, smem_addr + slot_off);
        } else {
#pragma unroll
            for (int j = 0; j < W::kPieces; ++j) {
                char *lk = smem + slot_off + j * 1024;
                const unsigned goff = goffp[j % W::kG] + j * 1024;   // my byte offset inside the tile in global memory
                if (page_ok && j * W::kRPI + lrow < rows_left) {
                    lds_dma16(kb, goff, smem_addr + slot_off + j * 1024);
                    lds_dma16(vb, goff, smem_addr + slot_off + j * 1024 + W::kKT);
                } else {
                    // past the end of the sequence (or a bad page id): the slot must not keep stale
                    // bits, since 0 * NaN would poison the row sums
                    *(uint4 *)(lk + lane * 16) = uint4{0u, 0u, 0u, 0u};
                    *(uint4 *)(lk + W::kKT + lane * 16) = uint4{0u, 0u, 0u, 0u};
                }
            }
        }
    };

        for (int t = 0; t < NS - 1; ++t)
            if (t < ntiles && wave == (t & (kWaves - 1))) issue(t, __builtin_amdgcn_readfirstlane(page_lds[t]), t);
        // the first tile this wavefront requests inside the loop: NS-1 .. NS+2, whichever is its turn
        int next_request = NS - 1 + ((wave - (NS - 1)) & (kWaves - 1));
        int next_page = next_request < ntiles ? page_lds[next_request] : -1;
        int slot_cur = 0;                                    // ring slot of tile t (t mod NS, kept incrementally)
        for (int t = 0; t < ntiles; ++t, slot_cur = (slot_cur + 1 == NS) ? 0 : slot_cur + 1) {
            if (wave == (t & (kWaves - 1))) wait_vmcnt0();   // the tile I fetched has landed
            __syncthreads();                                 // tile t visible; everyone is done with tile t-1
            const int tn = t + NS - 1;                       // goes into the slot tile t-1 occupied

            const int pos0 = c0 + t * kTile;
            const bool mask = pos0 + kTile > S - R;          // touches the new rows or the ragged end
            const int kx = slot_cur * W::kSlot + koff0, vx = slot_cur * W::kSlot + voff0;   // offsets in the ring
            // ---- S^T = K . Q^T
            const bool mine = XT && wave == (t & (kWaves - 1));      // my turn for the extra row tile
            f32x4 sacc[2][MT];
            f32x4 sx[2][1];
#pragma unroll
            for (int pt = 0; pt < 2; ++pt) {
#pragma unroll
                for (int rt = 0; rt < MT; ++rt) sacc[pt][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
                sx[pt][0] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            // K fragments one k-step ahead of the multiplications that use them
            bf16x8 kf[2][2];
#pragma unroll
            for (int pt = 0; pt < 2; ++pt) kf[0][pt] = *(const bf16x8 *)(smem + kx + pt * 16 * W::kRowBytes);
#pragma unroll
            for (int ks = 0; ks < D / 32; ++ks) {
                if (ks + 1 < D / 32) {
#pragma unroll
                    for (int pt = 0; pt < 2; ++pt)
                        kf[(ks + 1) & 1][pt] = *(const bf16x8 *)(smem + (kx ^ ((ks + 1) << 6)) + pt * 16 * W::kRowBytes);
                }
#pragma unroll
                for (int pt = 0; pt < 2; ++pt)
#pragma unroll
                    for (int rt = 0; rt < MT; ++rt)
                        sacc[pt][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[ks & 1][pt], w.qf[rt][ks], sacc[pt][rt], 0, 0, 0);
                if (mine) {
#pragma unroll
                    for (int pt = 0; pt < 2; ++pt)
                        sx[pt][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[ks & 1][pt], wx.qf[0][ks], sx[pt][0], 0, 0, 0);
                }
            }
            // The next tile is requested here rather than right after the barrier: the address arithmetic
            // and the load instructions of the fetching wavefront then run while its multiplications drain.
            if (tn < ntiles && wave == (tn & (kWaves - 1))) {
                issue(tn, __builtin_amdgcn_readfirstlane(next_page), slot_cur == 0 ? NS - 1 : slot_cur - 1);
                next_page = tn + kWaves < ntiles ? page_lds[tn + kWaves] : -1;
            }
            // ---- first half of the V fragments: issued now so their LDS latency hides under the softmax
            auto load_vf = [&](int dt) {
                const char *a0 = smem + (vx ^ (dt << 5));
                s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)a0);
                s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4 *)(a0 + 16 * W::kRowBytes));
                s16x8 cat = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                return __builtin_bit_cast(bf16x8, cat);
            };
            constexpr int kHalf = D / 32;
            bf16x8 vfa[kHalf];
#pragma unroll
            for (int i = 0; i < kHalf; ++i) vfa[i] = load_vf(i);
            __builtin_amdgcn_sched_barrier(0);               // keep the reads above the arithmetic below
            // The wavefront yields to the other workgroup's wavefront on this SIMD while it does its
            // softmax arithmetic and takes priority again for the matrix instructions: the two then tend
            // to alternate on the matrix pipe instead of both queueing for it.
            __builtin_amdgcn_s_setprio(0);
            // ---- softmax weights
            float c_eff = c;
            if ((sub == 0 && t == 0) || mask || raise_always) {   // rare: maxima, reference, masking
                float mx[MT];
                if (mask) softmax_max<D, MT, true>(w, sacc, mx, pos0, S, R, c, g);
                else softmax_max<D, MT, false>(w, sacc, mx, pos0, S, R, c, g);
#pragma unroll
                for (int rt = 0; rt < MT; ++rt)              // mx = -inf (nothing visible) leaves it unset
                    if (raise_always || w.m_run[rt] == kNegBig) w.m_run[rt] = fmaxf(w.m_run[rt], mx[rt]);
                if (mask) c_eff = 1.0f;                      // the masked form has scaled the scores in place
            }
            bf16x8 pf[MT];
            softmax_exp<D, MT, false>(w, sacc, c_eff, pf);   // fma(-inf, 1, -ref) = -inf -> weight 0
            bf16x8 pfx[1];
            if (mine) {
                if ((sub == 0 && t < kWaves) || mask || raise_always) {   // t < 4: my first extra tile of this pass
                    float mx1[1];
                    if (mask) softmax_max<D, 1, true>(wx, sx, mx1, pos0, S, R, c, g);
                    else softmax_max<D, 1, false>(wx, sx, mx1, pos0, S, R, c, g);
                    if (raise_always || wx.m_run[0] == kNegBig) wx.m_run[0] = fmaxf(wx.m_run[0], mx1[0]);
                }
                softmax_exp<D, 1, false>(wx, sx, c_eff, pfx);
            }
            __builtin_amdgcn_s_setprio(1);
            // ---- O^T += V^T . P^T ; the second half of V is fetched while the first is multiplied
            bf16x8 vfb[kHalf];
#pragma unroll
            for (int i = 0; i < kHalf; ++i) vfb[i] = load_vf(kHalf + i);
#pragma unroll
            for (int i = 0; i < kHalf; ++i)
#pragma unroll
                for (int rt = 0; rt < MT; ++rt)
                    w.oacc[i][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vfa[i], pf[rt], w.oacc[i][rt], 0, 0, 0);
#pragma unroll
            for (int i = 0; i < kHalf; ++i)
#pragma unroll
                for (int rt = 0; rt < MT; ++rt)
                    w.oacc[kHalf + i][rt] =
                        __builtin_amdgcn_mfma_f32_16x16x32_bf16(vfb[i], pf[rt], w.oacc[kHalf + i][rt], 0, 0, 0);
            if (mine) {
#pragma unroll
                for (int i = 0; i < kHalf; ++i) {
                    wx.oacc[i][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vfa[i], pfx[0], wx.oacc[i][0], 0, 0, 0);
                    wx.oacc[kHalf + i][0] =
                        __builtin_amdgcn_mfma_f32_16x16x32_bf16(vfb[i], pfx[0], wx.oacc[kHalf + i][0], 0, 0, 0);
                }
            }
        }

        __syncthreads();                                     // everyone is done with the ring before it refills
      }   // sub

        bool bad = false;
#pragma unroll
        for (int rt = 0; rt < MT; ++rt) bad = bad || !(w.l_part[rt] < 1.0e30f);    // also catches NaN
        if (XT) bad = bad || !(wx.l_part[0] < 1.0e30f);
        // Workgroup-wide OR through the first word of the (now idle) ring: the ring takes the whole
        // LDS share of a workgroup, so there is no room for a separate flag.
        if (tid == 0) *(volatile int *)smem = 0;
        __syncthreads();
        if (bad) *(volatile int *)smem = 1;
        __syncthreads();
        const bool redo = *(volatile int *)smem != 0;
        __syncthreads();                                     // everyone has read it before the ring refills
        if (attempt == 2 || (attempt == 0 && !redo)) break;
#pragma unroll
        for (int rt = 0; rt < MT; ++rt) {
            if (attempt == 0) w.m_run[rt] = kNegBig;         // attempt 1 finds the exact maxima from scratch
            w.l_part[rt] = 0.f;
#pragma unroll
            for (int dt = 0; dt < D / 16; ++dt) w.oacc[dt][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        if (XT) {
            if (attempt == 0) wx.m_run[0] = kNegBig;
            wx.l_part[0] = 0.f;
#pragma unroll
            for (int dt = 0; dt < D / 16; ++dt) wx.oacc[dt][0] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }

    // ---- every wavefront owns its rows outright: normalise (or leave a partial) straight from registers
    const int n_e = opaque(n), g_e = opaque(g), tid_e = opaque(tid);   // epilogue indices: computed here, not hoisted
    const bool final_out = sg.rec < 0;
    float *wo = nullptr, *wm = nullptr, *wl = nullptr;
    if (!final_out) {
        const int rpad = p.phase == 1 ? p.rows_pad_p : p.rows_pad;
        wo = (p.phase == 1 ? p.wsp : p.wsr) + sg.rec * ws_record_floats(rpad, D);
        wm = wo + (int64_t)rpad * D;
        wl = wm + rpad;
    }
#pragma unroll
    for (int rt = 0; rt < MT; ++rt) {
        float l = w.l_part[rt];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        const int pr = row0 + rt * 16 + n_e;
        if (pr < row_end) {
            if (final_out) {
                const int hh = pr / R, i = pr % R;
                const float inv = inv_or_zero(l);
                const int64_t o = (((int64_t)b * R + i) * p.Hq + (int64_t)kvh * p.G + hh) * D;
#pragma unroll
                for (int dt = 0; dt < D / 16; ++dt) {
                    const f32x4 a = w.oacc[dt][rt] * inv;
                    store_out(p.out, o + dt * 16 + 4 * g_e, float4{a[0], a[1], a[2], a[3]}, p.out_bf16);
                }
            } else {
#pragma unroll
                for (int dt = 0; dt < D / 16; ++dt) {
                    const f32x4 a = w.oacc[dt][rt];
                    *(float4 *)(wo + (int64_t)pr * D + dt * 16 + 4 * g_e) = float4{a[0], a[1], a[2], a[3]};
                }
                if (g_e == 0) { wm[pr] = w.m_run[rt]; wl[pr] = l; }
            }
        }
    }

    // ---- extra rows: each wavefront holds the contribution of the tiles it took; merge through LDS
    // (the ring is idle: the last barriers of the tile loop are behind every wavefront)
    if (XT) {
        float *xm = (float *)smem;                           // [4][16]
        float *xl = xm + kWaves * 16;                        // [4][16]
        float *xo = xl + kWaves * 16;                        // [16][D + 4]
        constexpr int kXStr = D + 4;
        float lx = wx.l_part[0];
        lx += __shfl_xor(lx, 16, 64);
        lx += __shfl_xor(lx, 32, 64);
        if (g_e == 0) { xm[wave * 16 + n_e] = wx.m_run[0]; xl[wave * 16 + n_e] = lx; }
        __syncthreads();
        float M = xm[n_e];
#pragma unroll
        for (int ww = 1; ww < kWaves; ++ww) M = fmaxf(M, xm[ww * 16 + n_e]);
        float L = 0.f;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) L += xl[ww * 16 + n_e] * __builtin_amdgcn_exp2f(xm[ww * 16 + n_e] - M);
        const float my_scale = __builtin_amdgcn_exp2f(wx.m_run[0] - M);
        for (int ww = 0; ww < kWaves; ++ww) {
            if (wave == ww) {
#pragma unroll
                for (int dt = 0; dt < D / 16; ++dt) {
                    float4 *dst = (float4 *)(xo + n_e * kXStr + dt * 16 + 4 * g_e);
                    const f32x4 a = wx.oacc[dt][0] * my_scale;
                    float4 v{a[0], a[1], a[2], a[3]};
                    if (ww > 0) { const float4 o = *dst; v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w; }
                    *dst = v;
                }
            }
            __syncthreads();
        }
        // every wavefront computed the same M and L; wavefront 0 publishes them over its own entries
        if (wave == 0 && g_e == 0) { xm[n_e] = M; xl[n_e] = L; }
        __syncthreads();
        const int rows_x = max(0, sg.rows - kXRow0);
        for (int idx = tid_e; idx < rows_x * (D / 4); idx += 256) {
            const int row = idx / (D / 4), c4 = idx % (D / 4);
            const int pr = kXRow0 + row;
            float4 v = *(const float4 *)(xo + row * kXStr + c4 * 4);
            if (final_out) {
                const int hh = pr / R, i = pr % R;
                const float inv = inv_or_zero(xl[row]);
                v.x *= inv; v.y *= inv; v.z *= inv; v.w *= inv;
                const int64_t o = (((int64_t)b * R + i) * p.Hq + (int64_t)kvh * p.G + hh) * D + c4 * 4;
                store_out(p.out, o, v, p.out_bf16);
            } else {
                *(float4 *)(wo + (int64_t)pr * D + c4 * 4) = v;
            }
        }
        if (!final_out && tid_e < rows_x) { wm[kXRow0 + tid_e] = xm[tid_e]; wl[kXRow0 + tid_e] = xl[tid_e]; }
    }
    __syncthreads();                                         // the ring is reused by the next segment
    });
}

template <int D, int MT, int NS, bool XT>
__global__ __launch_bounds__(256, 2) void attn_bf16_wide_kernel(const AttnParams p) {
    __shared__ __align__(16) char smem[NS * WideCfg<D>::kSlot];
    __shared__ int page_lds[kPageIds];
    __shared__ int sched_tmp[8];
    wide_body<D, MT, NS, XT>(p, smem, page_lds, sched_tmp, (int)blockIdx.x, (int)gridDim.x);
}

// Shared-prefix ("cascade") run in one launch.  Every workgroup has a share of the prefix phase (the wide
// body over the packed rows of a whole group of sessions: bound by the matrix and softmax arithmetic)
// and a share of the sessions' own parts (the wide body over one session's rows: bound by memory).
// Even workgroups take the prefix share first, odd ones the own-part share, and a compute unit holds one
// of each, so its matrix pipe and its memory stream are both busy for most of the launch, and every
// workgroup has the same total work: no tail.
template <int D, int MTP, bool XTP, int NS>
__global__ __launch_bounds__(256, 2) void attn_cascade_fused_kernel(const AttnParams p) {
    __shared__ __align__(16) char smem[NS * WideCfg<D>::kSlot];
    __shared__ int page_lds[kPageIds];
    __shared__ int sched_tmp[8];
    const int wg = (int)blockIdx.x, nwg = (int)gridDim.x;
#pragma nounroll
    for (int step = 0; step < 2; ++step) {
        if (((step ^ wg) & 1) == 0) {
            AttnParams pp = p;
            pp.phase = 1;
            pp.rows = p.gs * p.rows1;                        // rows1 stays the rows of one session
            pp.balanced = 0;
            wide_body<D, MTP, NS, XTP>(pp, smem, page_lds, sched_tmp, wg, nwg);
        } else {
            wide_body<D, 1, NS, false>(p, smem, page_lds, sched_tmp, wg, nwg);
        }
        __syncthreads();
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
    const int S = session_len(p, b);
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
        const float inv = inv_or_zero(L);
        acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
        const int hh = pr / p.R, i = pr % p.R;
        const int64_t o = (((int64_t)b * p.R + i) * p.Hq + (int64_t)ho * G_eff + hh) * D + c4 * 4;
        store_out(p.out, o, acc, p.out_bf16);
    }
}

// The same merge for the balanced schedule: the partials of stream (b, kv head) are the records of
// the workgroups whose shares overlap it, found from the prefix sums workgroup 0 left in the plan.
// Workgroup i keeps the partial of its first segment in record 2i and that of its last in 2i+1.
template <int D>
__global__ __launch_bounds__(256) void attn_merge_balanced_kernel(const AttnParams p, int nslots) {
    constexpr int kRowsPerWg = 256 / (D / 4);                // one thread per (row, 4 output values)
    const int kvh = blockIdx.x, b = blockIdx.y, slab = blockIdx.z;
    const int nt_b = tiles_of(session_len(p, b));
    if (nt_b == 0) {                                         // an empty session: no workgroup had any of it
        if (slab == 0) zero_session_heads(p.out, p.out_bf16, b, p.R, p.Hq, D, kvh * p.G, p.G);
        return;
    }
    const int T = p.plan[p.B] * p.Hkv;
    const int share = balanced_share(T, nslots);
    const int g0 = p.plan[b] * p.Hkv + kvh * nt_b, g1 = g0 + nt_b;      // the stream's place in the sequence
    const int i0 = g0 / share, i1 = (g1 - 1) / share;
    if (i0 == i1) return;                                    // one workgroup had all of it and wrote the output
    const int64_t recf = ws_record_floats(p.rows_pad, D);
    // the stream's piece is the first segment of every workgroup but possibly the first one
    const int first_slot = (i0 * share < g0) ? 1 : 0;
    auto record = [&](int i) { return p.wsr + (2 * (int64_t)i + (i == i0 ? first_slot : 0)) * recf; };
    const int pr = slab * kRowsPerWg + (int)threadIdx.x / (D / 4), c4 = (int)threadIdx.x % (D / 4);
    if (pr >= p.rows) return;
    float M = kNegBig;
    for (int i = i0; i <= i1; ++i) M = fmaxf(M, record(i)[(int64_t)p.rows_pad * D + pr]);
    float L = 0.f;
    float4 acc{0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int i = i0; i <= i1; ++i) {
        const float *rec = record(i);
        const float w = exp2f(rec[(int64_t)p.rows_pad * D + pr] - M);
        L += w * rec[(int64_t)p.rows_pad * D + p.rows_pad + pr];
        const float4 o = *(const float4 *)(rec + (int64_t)pr * D + c4 * 4);
        acc.x += w * o.x; acc.y += w * o.y; acc.z += w * o.z; acc.w += w * o.w;
    }
    const float inv = inv_or_zero(L);
    acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
    const int hh = pr / p.R, i = pr % p.R;
    const int64_t o = (((int64_t)b * p.R + i) * p.Hq + (int64_t)kvh * p.G + hh) * D + c4 * 4;
    store_out(p.out, o, acc, p.out_bf16);
}

// ------------------------------------------------------------------------------------------
// Shared-prefix ("cascade") runs.
//
// attn_lcp_kernel: lcp[b] = number of leading pages session b lists exactly as session 0 does, cut to
// the pages that lie wholly in front of the session's R new rows (so no row of any session is masked
// inside the shared prefix).  The minimum over the batch is the prefix every session shares.
// attn_merge_cascade_kernel: per (session, kv head), the log-sum-exp merge of the prefix records of the
// session's group (its rows are a slice of the group's packed rows) with the records of its own part.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void attn_lcp_kernel(const AttnParams p, int32_t *lcp) {
    __shared__ int tmp[4];
    const int b = blockIdx.x;
    const int usable_b = max(0, session_len(p, b) - p.R) / p.P;
    const int usable_0 = max(0, session_len(p, 0) - p.R) / p.P;
    const int n = min(usable_b, usable_0);
    const int32_t *rb = p.bt + (int64_t)b * p.max_pages, *r0 = p.bt;
    int first_bad = n;
    for (int j = threadIdx.x; j < n; j += 256) {
        const int pg = rb[j];
        if (pg != r0[j] || pg < 0 || (int64_t)pg >= p.num_pages) { first_bad = j; break; }   // j only grows
    }
    const int m = block_min(first_bad, tmp);
    if (threadIdx.x == 0) lcp[b] = m;
}

template <int D>
__global__ __launch_bounds__(256) void attn_merge_cascade_kernel(const AttnParams p) {
    __shared__ int tmp[4];
    constexpr int kRowsPerWg = 256 / (D / 4);                // one thread per (row, 4 output values)
    const int kvh = blockIdx.x, b = blockIdx.y, slab = blockIdx.z;
    const int ptiles = shared_prefix_tiles(p, tmp);
    const int nt_b = max(0, tiles_of(session_len(p, b)) - ptiles);
    if (nt_b == 0) {                                         // an empty session (a valid one has its new rows after the prefix)
        if (slab == 0) zero_session_heads(p.out, p.out_bf16, b, p.R, p.Hq, D, kvh * p.G, p.G);
        return;
    }
    // the session's own part: the records of the workgroups whose shares overlap the stream, or the stream's
    // own record when one workgroup had all of it
    const int T = p.plan[p.B] * p.Hkv;
    const int share = balanced_share(T, p.nslots);
    const int g0 = p.plan[b] * p.Hkv + kvh * nt_b, g1 = g0 + nt_b;
    const int i0 = g0 / share, i1 = (g1 - 1) / share;
    if (ptiles == 0 && i0 == i1) return;                     // no prefix part, one workgroup had the stream: output written
    const int64_t recf = ws_record_floats(p.rows_pad, D);
    const int64_t recfp = ws_record_floats(p.rows_pad_p, D);
    const int n_own = i1 - i0 + 1;
    auto own = [&](int j) { return p.wsr + ((int64_t)(i0 + j) + (int64_t)b * p.Hkv + kvh) * recf; };
    // the prefix part: the same arithmetic over the (group, kv head) streams of ptiles tiles each; the
    // session's rows are the slice [so*rows1, (so+1)*rows1) of its group's packed rows
    const int grp = b / p.gs, so = b % p.gs;
    int n_pre = 0, j0 = 0;
    const int sp = grp * p.Hkv + kvh;
    if (ptiles > 0) {
        const int share_p = balanced_share(p.ngroups * p.Hkv * ptiles, p.nslots);
        const int q0 = sp * ptiles, q1 = q0 + ptiles;
        j0 = q0 / share_p;
        n_pre = (q1 - 1) / share_p - j0 + 1;
    }
    auto pre = [&](int j) { return p.wsp + ((int64_t)(j0 + j) + sp) * recfp; };
    const int rows1 = p.rows1;
    const int pr = slab * kRowsPerWg + (int)threadIdx.x / (D / 4), c4 = (int)threadIdx.x % (D / 4);
    if (pr >= rows1) return;
    const int prp = so * rows1 + pr;
    // pass 1: the common reference; pass 2: the weighted sums (independent loads, several in flight)
    float M = kNegBig;
    for (int j = 0; j < n_own; ++j) M = fmaxf(M, own(j)[(int64_t)p.rows_pad * D + pr]);
    for (int j = 0; j < n_pre; ++j) M = fmaxf(M, pre(j)[(int64_t)p.rows_pad_p * D + prp]);
    float L = 0.f;
    float4 acc{0.f, 0.f, 0.f, 0.f};
    auto add = [&](const float *rec, int rpad, int row) {
        const float w = exp2f(rec[(int64_t)rpad * D + row] - M);
        const float l = rec[(int64_t)rpad * D + rpad + row];
        const float4 o = *(const float4 *)(rec + (int64_t)row * D + c4 * 4);
        L += w * l;
        acc.x += w * o.x; acc.y += w * o.y; acc.z += w * o.z; acc.w += w * o.w;
    };
#pragma unroll 4
    for (int j = 0; j < n_own; ++j) add(own(j), p.rows_pad, pr);
#pragma unroll 4
    for (int j = 0; j < n_pre; ++j) add(pre(j), p.rows_pad_p, prp);
    const float inv = inv_or_zero(L);
    acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
    const int hh = pr / p.R, i = pr % p.R;
    const int64_t o = (((int64_t)b * p.R + i) * p.Hq + (int64_t)kvh * p.G + hh) * D + c4 * 4;
    store_out(p.out, o, acc, p.out_bf16);
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
    const int S = session_len(p, b);
    const int c0 = chunk * p.chunk;
    if (S <= 0 && chunk == 0) zero_session_heads(p.out, p.out_bf16, b, p.R, p.Hq, D, h, 1);
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
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;   // wave index lives in an SGPR
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
            const float r = acc * inv_or_zero(row_l[i]);
            const int64_t o = (((int64_t)b * R + i) * p.Hq + h) * D + d;
            if (p.out_bf16) ((__hip_bfloat16 *)p.out)[o] = __float2bfloat16(r);
            else ((float *)p.out)[o] = r;
        }
    }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
struct Tuning {
    int sched;               // 0 auto, 1 chunk grid, 2 balanced
    int casc;                // 0 auto, 1 never, 2 look for a shared prefix
    int64_t kv_chunk;        // 0 auto, else KV positions per workgroup of the chunk grid
};

int parse_tuning(uint64_t word, Tuning *t) {
    t->sched = (int)(word & 3);
    t->casc = (int)((word >> 2) & 3);
    t->kv_chunk = (int64_t)((word >> 8) & 0xffffff) * 128;
    if (t->sched == 3 || t->casc == 3 || (word >> 32) != 0 || (word & 0xf0) != 0) return AGENTSAM_ERR_ARG;
    if (t->kv_chunk > (1ll << 30)) return AGENTSAM_ERR_ARG;
    return AGENTSAM_OK;
}

struct Plan {
    int chunk, nchunks_max, rows_pad, heads_outer;
    bool wide;
    bool balanced;           // balanced partition over `nslots` workgroups instead of the chunk grid
    int nslots;
    size_t plan_bytes;       // balanced: the prefix sums in front of the records
    size_t ws_bytes;
    // shared-prefix run
    bool cascade;
    int gs, ngroups, rows_group, rows_pad_p;
    size_t lcp_bytes, own_bytes; // workspace: [lcp][plan][own records][prefix records]
};

// Workgroups an MI355X keeps resident at once: 256 compute units x 2 (wide kernel, 68 KB of LDS and
// <= 256 registers) or x 1 (narrow kernel, which takes the whole register file of a SIMD).
constexpr int kComputeUnits = 256;

int make_plan(int B, int R, int Hq, int Hkv, int D, int page_size, int max_pages, int dtype, uint64_t tuning, Plan *pl) {
    if (B < 0 || R < 1 || Hq < 1 || Hkv < 1 || page_size < 1 || max_pages < 1) return AGENTSAM_ERR_ARG;
    if (Hq % Hkv != 0) return AGENTSAM_ERR_ARG;
    if (D != 64 && D != 128) return AGENTSAM_ERR_UNSUPPORTED;
    if (dtype != AGENTSAM_F32 && dtype != AGENTSAM_BF16) return AGENTSAM_ERR_UNSUPPORTED;
    Tuning tn;
    if (const int rc = parse_tuning(tuning, &tn)) return rc;
    const int64_t smax = (int64_t)max_pages * page_size;
    if (smax > 0x7fffff00ll) return AGENTSAM_ERR_ARG;
    const int G = Hq / Hkv;
    const int64_t opt = tn.kv_chunk;
    pl->wide = false;
    pl->cascade = false;
    pl->balanced = false;
    pl->nslots = 0;
    pl->plan_bytes = 0;
    if (dtype == AGENTSAM_F32) {
        if (R > kF32MaxR) return AGENTSAM_ERR_UNSUPPORTED;
        pl->chunk = kF32Chunk;                               // fixed: the score tile lives in LDS
        pl->rows_pad = R;
        pl->heads_outer = Hq;
    } else {
        if (page_size % kTile != 0) return AGENTSAM_ERR_UNSUPPORTED;
        const int rows = G * R;
        if (rows > kWaves * kRowsPerGroup) return AGENTSAM_ERR_UNSUPPORTED;
        pl->wide = rows > kRowsPerGroup;
        pl->rows_pad = (rows + 3) & ~3;                      // keeps every record 16-byte aligned
        pl->heads_outer = Hkv;
        pl->nslots = kComputeUnits * (pl->wide ? 2 : 1);
        int64_t chunk = opt;
        if (chunk == 0) {
            // about one workgroup per resident slot when every session has the maximum length: a
            // single round of workgroups, each streaming for as long as possible
            const int64_t pairs = (int64_t)B * Hkv;
            chunk = smax * (pairs > 0 ? pairs : 1) / pl->nslots;
            chunk = (chunk + 127) / 128 * 128;
            if (chunk < 1024) chunk = 1024;
            if (chunk > 8192) chunk = 8192;
        }
        // chunks start on page boundaries (when a page fits) and span at most 256 tiles
        int64_t unit = 128;
        while (unit % page_size != 0 && unit < kMaxChunk) unit += 128;     // lcm(128, page_size) if it fits
        if (unit % page_size != 0) unit = 128;
        chunk = (chunk + unit - 1) / unit * unit;
        if (chunk > kMaxChunk) chunk = kMaxChunk / unit * unit;
        pl->chunk = (int)chunk;
        // With at least two (session, kv head) streams per resident workgroup the batch is cut into
        // equal shares; with fewer, every stream is split anyway and the chunk grid keeps sessions
        // that share a prefix in step.  Streams that fit one chunk also stay on the chunk grid: a workgroup
        // per stream writes its output directly, and the fixed cost of a share (the scan of the batch, a drain
        // and a merge through LDS per stream in it, the merge launch) is a third of the run at 4096 positions
        // (B = 64, 8 kv heads: 192 us against 260 us; equal at 8192).  An explicit chunk size asks for the chunk grid.
        const int64_t tiles_max = (int64_t)B * Hkv * ((smax + kTile - 1) / kTile);
        pl->balanced = tn.sched == 2 ||
                       (tn.sched == 0 && opt == 0 && (int64_t)B * Hkv >= 2 * (int64_t)pl->nslots && smax > kMaxChunk);
        if (pl->balanced && tiles_max > 0x7fffffffll) {
            if (tn.sched == 2) return AGENTSAM_ERR_ARG;
            pl->balanced = false;
        }
    }
    pl->nchunks_max = (int)((smax + pl->chunk - 1) / pl->chunk);
    const size_t rec_bytes = (size_t)pl->rows_pad * (D + 2) * sizeof(float);
    if (dtype == AGENTSAM_BF16) {
        // Shared-prefix run: groups of gs sessions (as many as fit the wide kernel's 192 packed rows) take
        // the common prefix together, in the same launch as the sessions' own parts (which then go through
        // the wide kernel body too: up to 64 packed rows per session).  Looked for by default only when the
        // detection (a small launch, about 5 us) is below half a percent of the time the K/V stream itself takes.
        const int rows1 = G * R;
        const int gs = std::min<int>(B, (kWaves * kRowsPerGroup) / rows1);
        const double kv_bytes = (double)smax * B * Hkv * 2.0 * D * 2.0;
        const int64_t tiles_max = (int64_t)B * Hkv * ((smax + kTile - 1) / kTile);
        if (gs >= 2 && rows1 <= 64 && gs * rows1 > kRowsPerGroup && tiles_max <= 0x7fffffffll && opt == 0 &&
            tn.sched != 1 && (tn.casc == 2 || (tn.casc == 0 && kv_bytes >= 11.0e9))) {
            pl->cascade = true;
            pl->balanced = true;                             // the sessions' own parts: balanced shares
            pl->wide = true;
            // two workgroups per compute unit, fewer when the batch cannot have 16 tiles for each
            pl->nslots = (int)std::min<int64_t>(2 * kComputeUnits, std::max<int64_t>(16, tiles_max / 16));
            pl->gs = gs;
            pl->ngroups = (B + gs - 1) / gs;
            pl->rows_group = gs * rows1;
            pl->rows_pad_p = (pl->rows_group + 3) & ~3;
        }
    }
    if (pl->cascade) {
        pl->lcp_bytes = ((size_t)B * sizeof(int32_t) + 255) & ~(size_t)255;
        pl->plan_bytes = (((size_t)B + 1) * sizeof(int32_t) + 255) & ~(size_t)255;
        pl->own_bytes = ((size_t)pl->nslots + (size_t)B * Hkv) * rec_bytes;
        pl->ws_bytes = pl->lcp_bytes + pl->plan_bytes + pl->own_bytes +
                       ((size_t)pl->nslots + (size_t)pl->ngroups * Hkv) * (size_t)pl->rows_pad_p * (D + 2) * sizeof(float);
    } else if (pl->balanced) {
        pl->plan_bytes = (((size_t)B + 1) * sizeof(int32_t) + 255) & ~(size_t)255;
        pl->ws_bytes = pl->plan_bytes + 2 * (size_t)pl->nslots * rec_bytes;
    } else {
        pl->ws_bytes = (size_t)B * pl->heads_outer * pl->nchunks_max * rec_bytes;
        if (pl->nchunks_max <= 1) pl->ws_bytes = 0;
    }
    return AGENTSAM_OK;
}

template <int D>
hipError_t launch_bf16(const AttnParams &p, bool wide, dim3 grid, hipStream_t st) {
    using agentsam::launch;
    if (wide) {
        const int rpw = (p.rows + kWaves - 1) / kWaves;
        const int mt = (rpw + 15) / 16;
        // two workgroups per compute unit, each with a ring of tile slots in 64 KB of LDS (and 4 KB for the tiles' places)
        constexpr int NS = 65536 / WideCfg<D>::kSlot;
        // 4 x 16 x (mt-1) rows owned outright plus at most one shared extra row tile, when that fits
        const int extra = p.rows - kWaves * 16 * (mt - 1);
        if (mt >= 2 && extra >= 1 && extra <= 16) {
            if (mt == 2) return launch((attn_bf16_wide_kernel<D, 1, NS, true>), grid, dim3(256), st, p);
            return launch((attn_bf16_wide_kernel<D, 2, NS, true>), grid, dim3(256), st, p);
        }
        if (mt == 1) return launch((attn_bf16_wide_kernel<D, 1, NS, false>), grid, dim3(256), st, p);
        if (mt == 2) return launch((attn_bf16_wide_kernel<D, 2, NS, false>), grid, dim3(256), st, p);
        return launch((attn_bf16_wide_kernel<D, 3, NS, false>), grid, dim3(256), st, p);
    }
    const int mt = (p.rows + 15) / 16;
    if (mt == 1) return launch((attn_bf16_narrow_kernel<D, 1>), grid, dim3(256), st, p);
    if (mt == 2) return launch((attn_bf16_narrow_kernel<D, 2>), grid, dim3(256), st, p);
    return launch((attn_bf16_narrow_kernel<D, 3>), grid, dim3(256), st, p);
}

// the fused shared-prefix launch: the prefix phase's kernel variant follows the group's packed rows
template <int D>
hipError_t launch_cascade(const AttnParams &p, int rows_group, dim3 grid, hipStream_t st) {
    using agentsam::launch;
    constexpr int NS = 65536 / WideCfg<D>::kSlot;
    const int rpw = (rows_group + kWaves - 1) / kWaves;
    const int mt = (rpw + 15) / 16;
    const int extra = rows_group - kWaves * 16 * (mt - 1);
    if (mt >= 2 && extra >= 1 && extra <= 16) {
        if (mt == 2) return launch((attn_cascade_fused_kernel<D, 1, true, NS>), grid, dim3(256), st, p);
        return launch((attn_cascade_fused_kernel<D, 2, true, NS>), grid, dim3(256), st, p);
    }
    if (mt == 1) return launch((attn_cascade_fused_kernel<D, 1, false, NS>), grid, dim3(256), st, p);
    if (mt == 2) return launch((attn_cascade_fused_kernel<D, 2, false, NS>), grid, dim3(256), st, p);
    return launch((attn_cascade_fused_kernel<D, 3, false, NS>), grid, dim3(256), st, p);
}

#define ATTN_TRY(expr)                                        \
    do {                                                      \
        if ((expr) != hipSuccess) return AGENTSAM_ERR_HIP;    \
    } while (0)

// Everything spec_verify_attn does once the workspace is known (shared with the entry point whose
// workspace is the library's own static array).
int run_attn(const void *q, const void *k_cache, const void *v_cache, const int32_t *block_table, int32_t max_pages,
             const int32_t *seq_lens, int32_t B, int32_t R, int32_t Hq, int32_t Hkv, int32_t D, int32_t page_size,
             int64_t num_pages, float scale, int32_t dtype, int32_t out_dtype, void *out, void *workspace,
             size_t workspace_bytes, const Plan &pl, hipStream_t st) {
    using agentsam::launch;
    if (!(scale > 0.f) || num_pages < 0 || (B > 0 && num_pages < 1)) return AGENTSAM_ERR_ARG;
    if (out_dtype != AGENTSAM_F32 && out_dtype != AGENTSAM_BF16) return AGENTSAM_ERR_UNSUPPORTED;
    if (B == 0) return AGENTSAM_OK;
    if (!q || !k_cache || !v_cache || !block_table || !seq_lens || !out) return AGENTSAM_ERR_NULL;
    if (pl.ws_bytes > 0 && !workspace) return AGENTSAM_ERR_NULL;
    if (workspace_bytes < pl.ws_bytes) return AGENTSAM_ERR_WORKSPACE;
    if (B > 65535 || pl.heads_outer > 65535) return AGENTSAM_ERR_ARG;

    AttnParams p;
    p.q = q; p.kc = k_cache; p.vc = v_cache; p.bt = block_table; p.seq = seq_lens; p.out = out;
    p.ws = (float *)workspace;
    p.B = B; p.R = R; p.Hq = Hq; p.Hkv = Hkv; p.G = Hq / Hkv; p.D = D; p.P = page_size; p.max_pages = max_pages;
    p.num_pages = num_pages;
    p.log2P = -1;
    for (int sft = 0; sft < 31; ++sft)
        if ((1 << sft) == page_size) p.log2P = sft;
    p.scale_log2 = scale * kLog2e;
    p.chunk = pl.chunk; p.nchunks_max = pl.nchunks_max;
    p.rows = p.G * R; p.rows_pad = pl.rows_pad;
    p.out_bf16 = (out_dtype == AGENTSAM_BF16);
    p.balanced = pl.balanced ? 1 : 0;
    p.plan = (int32_t *)workspace;
    p.wsr = (float *)((char *)workspace + pl.plan_bytes);
    p.cascade = 0; p.phase = 0; p.gs = 1; p.ngroups = B; p.rows1 = p.rows;
    p.rows_pad_p = pl.rows_pad; p.nslots = pl.nslots; p.lcp = nullptr; p.wsp = nullptr;

    if (pl.cascade) {
        // [lcp][plan][own records][prefix records]
        char *wsb = (char *)workspace;
        int32_t *lcp = (int32_t *)wsb;
        p.cascade = 1;
        p.lcp = lcp;
        p.plan = (int32_t *)(wsb + pl.lcp_bytes);
        p.wsr = (float *)(wsb + pl.lcp_bytes + pl.plan_bytes);
        p.wsp = (float *)(wsb + pl.lcp_bytes + pl.plan_bytes + pl.own_bytes);
        p.gs = pl.gs; p.ngroups = pl.ngroups;
        p.rows_pad_p = pl.rows_pad_p;
        ATTN_TRY(launch(attn_lcp_kernel, dim3((unsigned)B), dim3(256), st, p, lcp));
        // one launch for the prefix phase (the packed rows of a whole group) and the sessions' own parts
        ATTN_TRY(D == 64 ? launch_cascade<64>(p, pl.rows_group, dim3((unsigned)pl.nslots), st)
                         : launch_cascade<128>(p, pl.rows_group, dim3((unsigned)pl.nslots), st));
        const int slabs = (p.rows + (256 / (D / 4)) - 1) / (256 / (D / 4));
        dim3 mg((unsigned)Hkv, (unsigned)B, (unsigned)slabs);
        ATTN_TRY(D == 64 ? launch(attn_merge_cascade_kernel<64>, mg, dim3(256), st, p)
                         : launch(attn_merge_cascade_kernel<128>, mg, dim3(256), st, p));
        return AGENTSAM_OK;
    }

    if (dtype == AGENTSAM_F32) {
        dim3 grid((unsigned)pl.nchunks_max, (unsigned)Hq, (unsigned)B);
        ATTN_TRY(D == 64 ? launch(attn_f32_kernel<64>, grid, dim3(256), st, p) : launch(attn_f32_kernel<128>, grid, dim3(256), st, p));
        if (pl.nchunks_max > 1) {
            dim3 mg((unsigned)Hq, (unsigned)B);
            ATTN_TRY(D == 64 ? launch(attn_merge_kernel<64>, mg, dim3(256), st, p, (int)Hq, 1)
                             : launch(attn_merge_kernel<128>, mg, dim3(256), st, p, (int)Hq, 1));
        }
        return AGENTSAM_OK;
    }

    if ((int64_t)pl.nchunks_max * Hkv * B > 0x7fffffffll) return AGENTSAM_ERR_ARG;
    dim3 grid(pl.balanced ? (unsigned)pl.nslots : (unsigned)((int64_t)pl.nchunks_max * Hkv * B));
    ATTN_TRY(D == 64 ? launch_bf16<64>(p, pl.wide, grid, st) : launch_bf16<128>(p, pl.wide, grid, st));
    dim3 mg((unsigned)Hkv, (unsigned)B);
    if (pl.balanced) {
        const int slabs = (p.rows + (256 / (D / 4)) - 1) / (256 / (D / 4));
        dim3 mgb((unsigned)Hkv, (unsigned)B, (unsigned)slabs);
        ATTN_TRY(D == 64 ? launch(attn_merge_balanced_kernel<64>, mgb, dim3(256), st, p, pl.nslots)
                         : launch(attn_merge_balanced_kernel<128>, mgb, dim3(256), st, p, pl.nslots));
    } else if (pl.nchunks_max > 1) {
        ATTN_TRY(D == 64 ? launch(attn_merge_kernel<64>, mg, dim3(256), st, p, (int)Hkv, p.G)
                         : launch(attn_merge_kernel<128>, mg, dim3(256), st, p, (int)Hkv, p.G));
    }
    return AGENTSAM_OK;
}

}  // namespace

extern "C" int spec_verify_attn_workspace(int32_t B, int32_t R, int32_t Hq, int32_t Hkv, int32_t D,
                                          int32_t page_size, int32_t max_pages, int32_t dtype, uint64_t tuning,
                                          size_t *bytes) {
    if (!bytes) return AGENTSAM_ERR_NULL;
    Plan pl;
    const int rc = make_plan(B, R, Hq, Hkv, D, page_size, max_pages, dtype, tuning, &pl);
    if (rc) return rc;
    *bytes = pl.ws_bytes;
    return AGENTSAM_OK;
}

extern "C" int spec_verify_attn(const void *q, const void *k_cache, const void *v_cache,
                                const int32_t *block_table, int32_t max_pages, const int32_t *seq_lens,
                                int32_t B, int32_t R, int32_t Hq, int32_t Hkv, int32_t D, int32_t page_size,
                                int64_t num_pages, float scale, int32_t dtype, int32_t out_dtype,
                                void *out, void *workspace, size_t workspace_bytes, uint64_t tuning, void *stream) {
    Plan pl;
    const int rc = make_plan(B, R, Hq, Hkv, D, page_size, max_pages, dtype, tuning, &pl);
    if (rc) return rc;
    return run_attn(q, k_cache, v_cache, block_table, max_pages, seq_lens, B, R, Hq, Hkv, D, page_size, num_pages, scale,
                    dtype, out_dtype, out, workspace, workspace_bytes, pl, (hipStream_t)stream);
}

// ---- the entry point that allocates nothing, for callers that cannot (graph capture, tight loops)
namespace {
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];              // device address of `scratch`, per device

int static_workspace(void **ptr) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return AGENTSAM_ERR_HIP;
    void *pv = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!pv) {
        // every GPU holds its own copy of the array at its own address: ask with that device current
        if (hipGetSymbolAddress(&pv, HIP_SYMBOL(scratch)) != hipSuccess || !pv) return AGENTSAM_ERR_HIP;
        g_scratch_ptr[dev].store(pv, std::memory_order_release);   // (two threads racing here store the same value)
    }
    *ptr = pv;
    return AGENTSAM_OK;
}
}  // namespace

extern "C" int spec_verify_attn_static(const void *q, const void *k_cache, const void *v_cache,
                                       const int32_t *block_table, int32_t max_pages, const int32_t *seq_lens,
                                       int32_t B, int32_t R, int32_t Hq, int32_t Hkv, int32_t D, int32_t page_size,
                                       int64_t num_pages, float scale, int32_t dtype, int32_t out_dtype,
                                       void *out, uint64_t tuning, void *stream) {
    Plan pl;
    const int rc = make_plan(B, R, Hq, Hkv, D, page_size, max_pages, dtype, tuning, &pl);
    if (rc) return rc;
    if (pl.ws_bytes > (size_t)AGENTSAM_STATIC_WORKSPACE_BYTES) return AGENTSAM_ERR_WORKSPACE;
    void *ws = nullptr;
    if (const int rs = static_workspace(&ws)) return rs;
    // Nothing in the workspace has to start at zero: every record, prefix sum and page count a launch
    // reads was written earlier in the same call, so the previous call's contents are simply overwritten.
    return run_attn(q, k_cache, v_cache, block_table, max_pages, seq_lens, B, R, Hq, Hkv, D, page_size, num_pages, scale,
                    dtype, out_dtype, out, ws, (size_t)AGENTSAM_STATIC_WORKSPACE_BYTES, pl, (hipStream_t)stream);
}
