// HIP kernels of the SGNS trainer for gfx950 (MI355X) other than the window kernel: weight
// initialisation, the draw dump used by the parity tests, the reduction self-test; and the host-side
// launchers of all kernels.
#include "w2v_train_kernel.h"

namespace w2v {
namespace {

// ---------------------------------------------------------------------------------------------
// weight initialisation: syn0[i][j] = (u24/2^24 - 0.5)/d from the seed, syn1neg = 0, padding = 0
// ---------------------------------------------------------------------------------------------
__global__ void init_weights_kernel(float *syn0, float *syn1neg, uint32_t vocab, uint32_t dim, uint32_t ld, uint64_t k0)
{
    const uint64_t n = (uint64_t)vocab * ld;
    for (uint64_t x = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; x < n; x += (uint64_t)gridDim.x * blockDim.x) {
        const uint64_t i = x / ld, j = x % ld;
        float v = 0.0f;
        if (j < dim) {
            const uint32_t u = (uint32_t)(mix64(k0 + (i * dim + j)) >> 32);
            v = (float)(((double)(u >> 8) * (1.0 / 16777216.0) - 0.5) / (double)dim);
        }
        syn0[x] = v;
        syn1neg[x] = 0.0f;
    }
}

__global__ void reset_accum_kernel(Accum *a, int what)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        a->next_sentence = 0;
        if (what >= 2) { a->loss_sum = 0.0; a->pairs = 0; a->dropped = 0; a->kept = 0; }
    }
}

// ---------------------------------------------------------------------------------------------
// draw dump: the integer decisions of every token, one thread per token
// ---------------------------------------------------------------------------------------------
__global__ void draws_kernel(KernelArgs A, uint64_t n_tokens, uint8_t *keep, uint8_t *width, int32_t *neg)
{
    for (uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; t < n_tokens; t += (uint64_t)gridDim.x * blockDim.x) {
        const int32_t w = A.tokens[t];
        const uint64_t base = position_base(A.key, A.first_pos + t);
        bool k = w >= 0 && (uint32_t)w < A.vocab;
        if (k) k = keep_decision(base, A.subsample ? A.thr[w] : 0xFFFFFFFFu);
        keep[t] = k ? 1 : 0;
        width[t] = k ? (uint8_t)window_width(base, A.window, A.window_mode) : 0;
        uint64_t nbase = base;
        if (k && A.neg_shift) {
            // sentence of token t: the last s with sent_off[s] <= t; its negatives come from the first position
            // of the stretch of 2^neg_shift tokens (counted from the sentence start) that t lies in
            uint64_t lo = 0, hi = A.n_sent;
            while (hi - lo > 1) {
                const uint64_t mid = lo + (hi - lo) / 2;
                if (A.sent_off[mid] <= t) lo = mid; else hi = mid;
            }
            const uint64_t start = A.sent_off[lo];
            nbase = position_base(A.key, A.first_pos + start + (((t - start) >> A.neg_shift) << A.neg_shift));
        }
        for (uint32_t j = 0; j < A.negatives; ++j)
            neg[t * A.negatives + j] = k ? A.table[negative_slot(nbase, j, A.table_size)] : -1;
    }
}

__global__ void __launch_bounds__(kLanes) reduce_selftest_kernel(const float *in, float *out)
{
    float v[CC * KC];
#pragma unroll
    for (int m = 0; m < CC * KC; ++m) v[m] = in[m * kLanes + threadIdx.x];
    out[threadIdx.x] = transpose_reduce<CC * KC>(v, threadIdx.x);
}

}  // namespace

TrainFn train_fn_v1r1k0(uint32_t window, bool full);
TrainFn train_fn_v1r1k1(uint32_t window, bool full);
TrainFn train_fn_v1r1k2(uint32_t window, bool full);
TrainFn train_fn_v1r1k3(uint32_t window, bool full);
TrainFn train_fn_v2r1k0(uint32_t window, bool full);
TrainFn train_fn_v2r1k1(uint32_t window, bool full);
TrainFn train_fn_v2r1k2(uint32_t window, bool full);
TrainFn train_fn_v2r1k3(uint32_t window, bool full);
TrainFn train_fn_v4r1k0(uint32_t window, bool full);
TrainFn train_fn_v4r1k1(uint32_t window, bool full);
TrainFn train_fn_v4r1k2(uint32_t window, bool full);
TrainFn train_fn_v4r1k3(uint32_t window, bool full);
TrainFn train_fn_v4r1t1k0(uint32_t window, bool full);
TrainFn train_fn_v4r1t1k1(uint32_t window, bool full);
TrainFn train_fn_v4r1t1k2(uint32_t window, bool full);
TrainFn train_fn_v4r1t1k3(uint32_t window, bool full);
TrainFn train_fn_v4r1t4k0(uint32_t window, bool full);
TrainFn train_fn_v4r1t4k1(uint32_t window, bool full);
TrainFn train_fn_v4r1t4k2(uint32_t window, bool full);
TrainFn train_fn_v4r1t4k3(uint32_t window, bool full);
TrainFn train_fn_v1r5k0(uint32_t window, bool full);
TrainFn train_fn_v1r5k1(uint32_t window, bool full);
TrainFn train_fn_v1r5k2(uint32_t window, bool full);
TrainFn train_fn_v1r5k3(uint32_t window, bool full);
TrainFn train_fn_v4r2k0(uint32_t window, bool full);
TrainFn train_fn_v4r2k1(uint32_t window, bool full);
TrainFn train_fn_v4r2k2(uint32_t window, bool full);
TrainFn train_fn_v4r2k3(uint32_t window, bool full);

namespace {
TrainFn train_fn(const KernelArgs &a, RowShape s)
{
    const bool full = a.dim == (uint32_t)(kLanes * floats_per_lane(s));
    const uint32_t rows = a.negatives + 1;                  // output rows of a window
    const int kmode = rows > 2u * KC ? 3 : rows > (uint32_t)KC ? 2 : rows == (uint32_t)KC ? 1 : 0;
#define W2V_PICK(VW, R)                                                                              \
    if (s.vw == VW && s.r == R && s.tail == 0)                                                       \
        return kmode == 3 ? train_fn_v##VW##r##R##k3(a.window, full)                                 \
             : kmode == 2 ? train_fn_v##VW##r##R##k2(a.window, full)                                 \
             : kmode == 1 ? train_fn_v##VW##r##R##k1(a.window, full) : train_fn_v##VW##r##R##k0(a.window, full);
    if (s.vw == 4 && s.r == 1 && s.tail == 1)
        return kmode == 3 ? train_fn_v4r1t1k3(a.window, full) : kmode == 2 ? train_fn_v4r1t1k2(a.window, full)
             : kmode == 1 ? train_fn_v4r1t1k1(a.window, full) : train_fn_v4r1t1k0(a.window, full);
    if (s.vw == 4 && s.r == 1 && s.tail == 4)
        return kmode == 3 ? train_fn_v4r1t4k3(a.window, full) : kmode == 2 ? train_fn_v4r1t4k2(a.window, full)
             : kmode == 1 ? train_fn_v4r1t4k1(a.window, full) : train_fn_v4r1t4k0(a.window, full);
    W2V_PICK(1, 1)
    W2V_PICK(2, 1)
    W2V_PICK(4, 1)
    W2V_PICK(1, 5)
    W2V_PICK(4, 2)
#undef W2V_PICK
    return nullptr;
}
}  // namespace

// ---------------------------------------------------------------------------------------------
// host side of the kernels
// ---------------------------------------------------------------------------------------------
bool pick_row_shape(uint32_t dim, uint32_t ld, RowShape *out)
{
    // by floats per lane; a row of 260..320 floats is one 16-byte chunk plus one float per lane when its length
    // allows (a quarter of the memory instructions of five single floats).  A chunk of several floats is
    // range-checked as a whole, so it must not straddle the end of a row: the length is a multiple of the
    // chunk, or (shapes with single floats behind the chunks) the chunks end inside the row.
    static const RowShape shapes[] = {{1, 1, 0}, {2, 1, 0}, {4, 1, 0}, {4, 1, 1}, {1, 5, 0}, {4, 2, 0}, {4, 1, 4}};
    for (const RowShape &s : shapes) {
        if ((uint32_t)(kLanes * floats_per_lane(s)) < dim) continue;
        const bool chunks_inside = s.tail > 1 && dim >= (uint32_t)(kLanes * s.vw * s.r);
        if ((dim % s.vw && !chunks_inside) || ld % s.vw) continue;
        *out = s;
        return true;
    }
    return false;
}

uint32_t train_lds_bytes(const KernelArgs &a, RowShape s)
{
    const uint32_t rowf = kLanes * floats_per_lane(s);
    return (2 * a.window + 3) * rowf * 4u + FCAP * 8u + kLanes * 32u + kLanes * a.negatives * 4u;
}

hipError_t launch_init_weights(float *syn0, float *syn1neg, uint32_t vocab, uint32_t dim, uint32_t ld,
                               uint64_t seed, hipStream_t stream)
{
    const uint64_t n = (uint64_t)vocab * ld;
    const uint32_t blocks = (uint32_t)((n + 255) / 256 < 8192 ? (n + 255) / 256 : 8192);
    hipLaunchKernelGGL(init_weights_kernel, dim3(blocks), dim3(256), 0, stream, syn0, syn1neg, vocab, dim, ld,
                       mix64(seed ^ 0x696E6974ull));
    return hipGetLastError();
}

hipError_t launch_reset_accum(Accum *accum, int what, hipStream_t stream)
{
    hipLaunchKernelGGL(reset_accum_kernel, dim3(1), dim3(64), 0, stream, accum, what);
    return hipGetLastError();
}

uint32_t train_resident_waves(const KernelArgs &a, int device)
{
    RowShape s;
    if (!pick_row_shape(a.dim, a.ld, &s)) return 0;
    TrainFn fn = train_fn(a, s);
    if (!fn) return 0;
    int per_cu = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kLanes, train_lds_bytes(a, s)) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) return 0;
    return (uint32_t)(per_cu > 0 ? per_cu : 1) * (uint32_t)(cus > 0 ? cus : 1);
}

hipError_t launch_train(const KernelArgs &a, uint32_t waves, hipStream_t stream)
{
    RowShape s;
    if (!pick_row_shape(a.dim, a.ld, &s)) return hipErrorInvalidValue;
    TrainFn fn = train_fn(a, s);
    if (!fn) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fn, dim3(waves), dim3(kLanes), train_lds_bytes(a, s), stream, a);
    return hipGetLastError();
}

hipError_t launch_draws(const KernelArgs &a, uint64_t n_tokens, uint8_t *keep, uint8_t *width, int32_t *neg,
                        hipStream_t stream)
{
    if (n_tokens == 0) return hipSuccess;
    const uint32_t blocks = (uint32_t)((n_tokens + 255) / 256 < 16384 ? (n_tokens + 255) / 256 : 16384);
    hipLaunchKernelGGL(draws_kernel, dim3(blocks), dim3(256), 0, stream, a, n_tokens, keep, width, neg);
    return hipGetLastError();
}

hipError_t launch_reduce_selftest(const float *in, float *out, hipStream_t stream)
{
    hipLaunchKernelGGL(reduce_selftest_kernel, dim3(1), dim3(kLanes), 0, stream, in, out);
    return hipGetLastError();
}

}  // namespace w2v
