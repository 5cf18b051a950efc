// No-reuse comparator of the window kernel: same sampling decisions, but every (target, context)
// pairing goes through global memory in the classic word2vec order -- for each context word, read its
// syn0 row; for each of the N+1 samples read the syn1neg row, take the dot product, update and write
// the row back at once; then write the context row back.  (2N+4) row transfers per pairing instead of
// (2N+4) per window: the role the pre-existing GPU kernels play in Table 4 of the paper.  It exists to
// measure memory traffic against w2v_train_epoch, not to be fast.
//
// One wavefront per sentence (work queue).  A sentence longer than kPiece tokens is handled in pieces of
// kPiece tokens, each treated as a sentence of its own (context does not cross a piece boundary).
#include "w2v_internal.h"
#include "w2v_rng.h"

namespace w2v {
namespace {

constexpr int kLanes = 64;
constexpr int kPiece = 1024;          // tokens compacted at once
constexpr int kMaxChunks = 8;         // 8 * 64 floats = W2V_MAX_DIM
constexpr int kMaxNeg = 20;

__device__ __forceinline__ uint32_t uni(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ uint64_t uni64(uint64_t v)
{
    return ((uint64_t)uni((uint32_t)(v >> 32)) << 32) | uni((uint32_t)v);
}
__device__ __forceinline__ float wave_sum_f(float x)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, kLanes);
    return x;
}
__device__ __forceinline__ double wave_sum_d(double x)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, kLanes);
    return x;
}

__global__ void __launch_bounds__(kLanes) naive_kernel(KernelArgs A)
{
    __shared__ int32_t kw[kPiece];
    __shared__ uint32_t kp[kPiece];
    __shared__ int32_t negs[kMaxNeg + 1];
    const int lane = threadIdx.x;
    const uint32_t W = A.window, N = A.negatives, d = A.dim;
    double loss_acc = 0.0;
    unsigned long long pairs_acc = 0, kept_acc = 0, dropped_acc = 0;

    for (;;) {
        unsigned long long s_raw = 0;
        if (lane == 0) s_raw = atomicAdd(&A.accum->next_sentence, 1ull);
        const uint64_t s = uni64(s_raw);
        if (s >= A.n_sent) break;
        const uint64_t t0 = uni64(A.sent_off[s]);
        const uint64_t t1 = uni64(A.sent_off[s + 1]);
        const uint64_t len = t1 > t0 ? t1 - t0 : 0;
        double frac = 1.0 - (double)(A.lr_done_base + A.first_pos + t0) / (double)A.lr_all;
        if (frac < A.lr_min_frac) frac = A.lr_min_frac;
        const float alpha = (float)(A.lr0 * frac);

        for (uint64_t piece = 0; piece < len; piece += kPiece) {
            const uint32_t plen = (uint32_t)((len - piece < (uint64_t)kPiece) ? len - piece : (uint64_t)kPiece);
            // kept tokens of the piece, in order
            uint32_t nk = 0;
            for (uint32_t base_off = 0; base_off < plen; base_off += kLanes) {
                const uint32_t off = base_off + lane;
                bool k = false;
                int32_t w = -1;
                if (off < plen) {
                    w = A.tokens[t0 + piece + off];
                    k = w >= 0 && (uint32_t)w < A.vocab;
                    if (!k) ++dropped_acc;
                    if (k && A.subsample) {
                        const uint32_t th = A.thr[w];
                        if (th != 0xFFFFFFFFu) k = keep_decision(position_base(A.key, A.first_pos + t0 + piece + off), th);
                    }
                }
                const uint64_t km = __ballot(k);
                if (k) {
                    const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(km >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)km, 0u));
                    kw[nk + rank] = w;
                    kp[nk + rank] = (uint32_t)(piece + off);
                }
                nk += (uint32_t)__popcll(km);
            }
            __syncthreads();
            kept_acc += nk;

            for (uint32_t i = 0; i < nk; ++i) {
                const int32_t center = kw[i];
                const uint64_t base = position_base(A.key, A.first_pos + t0 + kp[i]);
                const uint32_t b = window_width(base, W, A.window_mode);
                __syncthreads();
                if (lane == 0) negs[0] = center;
                if ((uint32_t)lane < N) negs[1 + lane] = A.table[negative_slot(base, (uint32_t)lane, A.table_size)];
                __syncthreads();
                const uint32_t lo = i > b ? i - b : 0u;
                const uint32_t hi = (i + b < nk) ? i + b : nk - 1u;
                for (uint32_t c = lo; c <= hi; ++c) {
                    if (c == i) continue;
                    float *irow = A.syn0 + (size_t)kw[c] * A.ld;
                    float I[kMaxChunks], neu[kMaxChunks];
#pragma unroll
                    for (int r = 0; r < kMaxChunks; ++r) {
                        const uint32_t e = (uint32_t)(r * kLanes + lane);
                        I[r] = e < d ? irow[e] : 0.0f;
                        neu[r] = 0.0f;
                    }
                    for (uint32_t k = 0; k <= N; ++k) {
                        const int32_t o = negs[k];
                        if (k >= 1 && o == center) continue;
                        float *orow = A.syn1neg + (size_t)o * A.ld;
                        float O[kMaxChunks];
                        float part = 0.0f;
#pragma unroll
                        for (int r = 0; r < kMaxChunks; ++r) {
                            const uint32_t e = (uint32_t)(r * kLanes + lane);
                            O[r] = e < d ? orow[e] : 0.0f;
                            part = __builtin_fmaf(I[r], O[r], part);
                        }
                        const float x = wave_sum_f(part);
                        const float sig = 1.0f / (1.0f + __expf(-x));
                        const float g = alpha * ((k == 0 ? 1.0f : 0.0f) - sig);
                        if (lane == 0) {
                            const float z = (k == 0) ? -x : x;
                            loss_acc += (double)(fmaxf(z, 0.0f) + __logf(1.0f + __expf(-fabsf(z))));
                        }
#pragma unroll
                        for (int r = 0; r < kMaxChunks; ++r) {
                            const uint32_t e = (uint32_t)(r * kLanes + lane);
                            neu[r] = __builtin_fmaf(g, O[r], neu[r]);
                            if (e < d) orow[e] = __builtin_fmaf(g, I[r], O[r]);
                        }
                    }
#pragma unroll
                    for (int r = 0; r < kMaxChunks; ++r) {
                        const uint32_t e = (uint32_t)(r * kLanes + lane);
                        if (e < d) irow[e] = I[r] + neu[r];
                    }
                    ++pairs_acc;
                }
            }
            __syncthreads();
        }
    }
    const double lsum = wave_sum_d(loss_acc);
    const unsigned long long dsum = (unsigned long long)wave_sum_d((double)dropped_acc);
    if (lane == 0) {
        atomicAdd(&A.accum->loss_sum, lsum);
        atomicAdd(&A.accum->pairs, pairs_acc);
        atomicAdd(&A.accum->kept, kept_acc);
        if (dsum) atomicAdd(&A.accum->dropped, dsum);
    }
}

}  // namespace

hipError_t launch_train_naive(const KernelArgs &a, uint32_t waves, hipStream_t stream)
{
    hipLaunchKernelGGL(naive_kernel, dim3(waves), dim3(kLanes), 0, stream, a);
    return hipGetLastError();
}

uint32_t naive_resident_waves(int device)
{
    int per_cu = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, naive_kernel, kLanes, 0) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) return 0;
    return (uint32_t)(per_cu > 0 ? per_cu : 1) * (uint32_t)(cus > 0 ? cus : 1);
}

}  // namespace w2v
