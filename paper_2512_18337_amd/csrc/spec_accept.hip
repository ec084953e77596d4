// spec_accept: greedy verification of the drafts.
//
// Alg. 4 (validation by the main model, commit of the matched prefix, fall-back at the first mismatch) and
// the losslessness claim of Sec. 5.4.1: the committed tokens equal greedy decoding.
//
// Two launches on the caller's stream:
//   1. row_argmax: one workgroup per logits row streams the row once with 16-byte loads
//      (the kernel is bound by HBM bandwidth: V*sizeof(logit) bytes per row, nothing reused)
//      and reduces (value, index) pairs with the first-index tie rule through wavefront
//      shuffles and one LDS exchange.
//   2. accept_prefix: one lane per session compares the drafts with the row targets.
//
// Two other arrangements were built, passed the same tests and were measured on the headline batch
// (576 rows of 128 KB; this arrangement: 16.7 us + 4.1 us):
//   - rows cut into segments, one workgroup per (row, segment), partial maxima in a scratch array, the
//     second launch taking the best segment per row: the first launch takes the same 16.6 us (at 74 MB
//     it is the ramp-up of the launch, not the number of workgroups, that keeps it from the streaming
//     rate) and the second twice as long;
//   - one launch, the last workgroup of a session to arrive doing step 2: merging a row maximum and
//     counting the arrival are two dependent device-scope atomic operations per workgroup, resolved at
//     the memory side, and the last arriver then has a chain of its own: 30 us; with memory fences,
//     which write back and invalidate an L2 on this GPU, 118 us.
#include <hip/hip_bf16.h>

#include "common.h"

namespace {

constexpr int kThreads = 256;
constexpr int kNoIndex = 0x7fffffff;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct Best {
    float v;
    int i;
};

// candidate b replaces a when it is larger, or equal with a lower index
__device__ __forceinline__ Best better(Best a, Best b) {
    const bool take = (b.v > a.v) || (b.v == a.v && b.i < a.i);
    return take ? b : a;
}

__device__ __forceinline__ float clean(float x) { return (x != x) ? -INFINITY : x; }   // NaN never wins

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

template <bool BF16>
__device__ __forceinline__ float load_one(const void *row, int64_t i) {
    if (BF16) return bf16_bits_to_float(((const uint16_t *)row)[i]);
    return ((const float *)row)[i];
}

// (value, index) of the first maximum of row[e0 .. e1), over the workgroup; valid in thread 0.
// index kNoIndex: nothing in the range is above -inf.
template <bool BF16>
__device__ __forceinline__ Best segment_argmax(const char *row, int64_t e0, int64_t e1) {
    constexpr int kElem = BF16 ? 2 : 4;
    constexpr int kPerVec = 16 / kElem;
    const int tid = threadIdx.x;
    // an unaligned head, a 16-byte-aligned body and a tail
    const char *seg = row + e0 * kElem;
    const int64_t n = e1 - e0;
    const int64_t mis = (int64_t)((uintptr_t)seg & 15);
    int64_t head = mis ? (16 - mis) / kElem : 0;
    if (head > n) head = n;
    const int64_t nvec = (n - head) / kPerVec;
    const int64_t tail0 = head + nvec * kPerVec;

    Best best{-INFINITY, kNoIndex};
    if (tid < head) {
        const float x = clean(load_one<BF16>(seg, tid));
        if (x > best.v) best = Best{x, (int)(e0 + tid)};
    }
    const u32x4 *body = (const u32x4 *)(seg + head * kElem);
#pragma unroll 4
    for (int64_t j = tid; j < nvec; j += kThreads) {
        const u32x4 w = __builtin_nontemporal_load(body + j);
        const int64_t base = e0 + head + j * kPerVec;
        const uint32_t ws[4] = {w[0], w[1], w[2], w[3]};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (BF16) {
                const float x0 = clean(bf16_bits_to_float(ws[c] & 0xffffu));
                const float x1 = clean(__uint_as_float(ws[c] & 0xffff0000u));
                if (x0 > best.v) best = Best{x0, (int)(base + 2 * c)};
                if (x1 > best.v) best = Best{x1, (int)(base + 2 * c + 1)};
            } else {
                const float x = clean(__uint_as_float(ws[c]));
                if (x > best.v) best = Best{x, (int)(base + c)};
            }
        }
    }
    // every thread visits its indices in increasing order (head < body < tail), so the strict
    // comparison keeps the first maximum it sees
    for (int64_t i = tail0 + tid; i < n; i += kThreads) {
        const float x = clean(load_one<BF16>(seg, i));
        if (x > best.v) best = Best{x, (int)(e0 + i)};
    }

#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        Best o{__shfl_xor(best.v, off, 64), __shfl_xor(best.i, off, 64)};
        best = better(best, o);
    }
    __shared__ float sv[kThreads / 64];
    __shared__ int si[kThreads / 64];
    if ((tid & 63) == 0) { sv[tid >> 6] = best.v; si[tid >> 6] = best.i; }
    __syncthreads();
    Best r{sv[0], si[0]};
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) r = better(r, Best{sv[w], si[w]});
    return r;
}

__device__ __forceinline__ void commit_session(int b, int k, const int32_t *tgt_row, const int32_t *__restrict__ draft,
                                               const int32_t *__restrict__ n_draft, int32_t *__restrict__ accept_len,
                                               int32_t *__restrict__ out_tokens) {
    // one lane: R <= 65 tokens
    const int R = k + 1;
    const int nd = min(max(n_draft[b], 0), k);
    int a = 0;
    while (a < nd && draft[(int64_t)b * k + a] == tgt_row[a]) ++a;
    accept_len[b] = a;
    for (int i = 0; i < R; ++i) out_tokens[(int64_t)b * R + i] = (i <= a) ? tgt_row[i] : -1;
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void row_argmax_kernel(const void *__restrict__ logits, int64_t V,
                                                              int32_t *__restrict__ tgt) {
    constexpr int kElem = BF16 ? 2 : 4;
    const int64_t row_id = blockIdx.x;
    const Best r = segment_argmax<BF16>((const char *)logits + row_id * V * kElem, 0, V);
    if (threadIdx.x == 0) tgt[row_id] = (r.i == kNoIndex) ? 0 : r.i;       // no finite maximum: index 0
}

__global__ void accept_prefix_kernel(const int32_t *__restrict__ tgt, const int32_t *__restrict__ draft,
                                     const int32_t *__restrict__ n_draft, int B, int k,
                                     int32_t *__restrict__ accept_len, int32_t *__restrict__ out_tokens) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    commit_session(b, k, tgt + (int64_t)b * (k + 1), draft, n_draft, accept_len, out_tokens);
}

}  // namespace

extern "C" int spec_accept(const void *logits, int32_t logits_dtype, const int32_t *draft,
                           const int32_t *n_draft, int32_t B, int32_t k, int64_t V,
                           int32_t *accept_len, int32_t *out_tokens, int32_t *tgt, void *stream) {
    if (B < 0 || k < 0 || k > 64 || V < 1 || V > 0x7ffffff0ll) return AGENTSAM_ERR_ARG;
    if (logits_dtype != AGENTSAM_F32 && logits_dtype != AGENTSAM_BF16) return AGENTSAM_ERR_UNSUPPORTED;
    if (B == 0) return AGENTSAM_OK;
    if (!logits || !n_draft || !accept_len || !out_tokens || !tgt || (k > 0 && !draft)) return AGENTSAM_ERR_NULL;
    const int64_t rows = (int64_t)B * (k + 1);
    if (rows > 0x7fffffffll) return AGENTSAM_ERR_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (logits_dtype == AGENTSAM_BF16) AGENTSAM_LAUNCH(row_argmax_kernel<true>, dim3((unsigned)rows), dim3(kThreads), st, logits, V, tgt);
    else AGENTSAM_LAUNCH(row_argmax_kernel<false>, dim3((unsigned)rows), dim3(kThreads), st, logits, V, tgt);
    AGENTSAM_LAUNCH(accept_prefix_kernel, dim3((unsigned)((B + 63) / 64)), dim3(64), st, tgt, draft, n_draft, (int)B,
                    (int)k, accept_len, out_tokens);
    return AGENTSAM_OK;
}
