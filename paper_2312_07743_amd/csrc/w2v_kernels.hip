// HIP kernels of the SGNS trainer for gfx950 (MI355X) other than the window kernel: weight
// initialisation, the draw dump used by the parity tests, the reduction self-test; and the host-side
// launchers of all kernels.
#include <mutex>

#include "w2v_train_kernel.h"

namespace w2v {

// Scratch memory of w2v_train_epoch_static (accumulators, work-queue head, ring snapshots of the summed mode): part of
// the code object, so no call allocates it; every GPU the library runs on holds its own copy until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress: kernels get the address asked for here.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

hipError_t static_scratch(int device, unsigned char **ptr)
{
    constexpr int kMaxDevices = 64;
    static std::mutex lock;
    static unsigned char *address[kMaxDevices] = {};
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(lock);
    if (!address[device]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        address[device] = static_cast<unsigned char *>(p);
    }
    *ptr = address[device];
    return hipSuccess;
}

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

// the same initial values rounded to the nearest bfloat16 (ties to even)
__global__ void init_weights_bf16_kernel(uint16_t *syn0, uint16_t *syn1neg, uint32_t vocab, uint32_t dim, uint32_t ld, uint64_t k0)
{
    const uint64_t n = (uint64_t)vocab * ld;
    for (uint64_t x = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; x < n; x += (uint64_t)gridDim.x * blockDim.x) {
        const uint64_t i = x / ld, j = x % ld;
        uint32_t b = 0;
        if (j < dim) {
            const uint32_t u = (uint32_t)(mix64(k0 + (i * dim + j)) >> 32);
            b = __float_as_uint((float)(((double)(u >> 8) * (1.0 / 16777216.0) - 0.5) / (double)dim));
            b += 0x7FFFu + ((b >> 16) & 1u);
        }
        syn0[x] = (uint16_t)(b >> 16);
        syn1neg[x] = 0;
    }
}

__global__ void widen_rows_kernel(const uint16_t *src, float *dst, uint32_t vocab, uint32_t dim, uint32_t ld)
{
    const uint64_t n = (uint64_t)vocab * dim;
    for (uint64_t x = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; x < n; x += (uint64_t)gridDim.x * blockDim.x)
        dst[x] = __uint_as_float((uint32_t)src[(x / dim) * ld + x % dim] << 16);
}

__global__ void reset_accum_kernel(Accum *a, int what)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        a->next_sentence = 0;
        if (what >= 2) { a->loss_sum = 0.0; a->pairs = 0; a->dropped = 0; a->kept = 0; }
    }
}

__global__ void export_accum_kernel(const Accum *a, double *loss_sum, uint64_t *pairs)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        if (loss_sum) *loss_sum = a->loss_sum;
        if (pairs) *pairs = a->pairs;
    }
}

// Cuts the launch's sentences into units of work and leaves the plan in the accumulator block.  A wavefront holds a
// unit until it is done, so there must be enough units that the wavefronts finish within a small fraction of the
// launch of one another; every unit re-reads the few tokens of context on either side, so units stay at 128 tokens
// or more on average.  Lock-free launches end the queue with units half that size (the last eighth of the
// sentences, at least 32 tokens on average).  (Measured on 17,000 sentences of 1,000 tokens: 250-token units 4 %
// faster than whole sentences, the finer end another 1.2 %; finer still loses to the context every unit re-reads.)
// The token count is that of this call, read from the offsets: a call that feeds part of an epoch is planned by
// its own size.  One wavefront (strict order) gains nothing from a finer queue.
__global__ void plan_kernel(Accum *a, const uint64_t *sent_off, PlanRequest rq)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const uint64_t n_sent = rq.n_sent;
    const uint64_t n_tokens = n_sent ? sent_off[n_sent] - sent_off[0] : 0;
    uint32_t shift = 0;
    if (rq.forced_unit_shift >= 0) shift = (uint32_t)rq.forced_unit_shift;
    else if (rq.waves > 1 && n_sent > 0)
        while (shift < 16 && (n_sent << shift) < 16u * rq.waves && (n_tokens / n_sent) >> (shift + 1) >= 128u) ++shift;
    uint32_t fine = shift;
    uint64_t coarse = n_sent;
    if (rq.forced_fine_shift >= 0) {
        fine = (uint32_t)rq.forced_fine_shift;
        coarse = rq.forced_coarse_sent < n_sent ? rq.forced_coarse_sent : n_sent;
    } else if (rq.forced_unit_shift < 0 && rq.waves > 1 && n_sent > 0) {
        if (fine < 16u && (n_tokens / n_sent) >> (fine + 1u) >= 32u) ++fine;
        if (fine > shift) coarse = n_sent - (n_sent / 8u ? n_sent / 8u : 1u);
    }
    a->unit_shift = shift;
    a->fine_shift = fine;
    a->coarse_sent = coarse;
    a->n_units = (coarse << shift) + ((n_sent - coarse) << fine);
    a->next_sentence = 0;
}

// test surface: defaults of the decision dump (a token that gets no window reads as dropped)
__global__ void fill_dump_kernel(DrawDump d, uint64_t n_tokens, uint32_t negatives)
{
    for (uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; t < n_tokens; t += (uint64_t)gridDim.x * blockDim.x) {
        d.keep[t] = 0;
        d.width[t] = 0;
        for (uint32_t k = 0; k < negatives; ++k) d.neg[t * negatives + k] = -1;
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

#include "w2v_train_table.inc"      // generated by build.py: one entry per instantiation unit that was built

namespace {
TrainFn train_fn(const KernelArgs &a, RowShape s, int update)
{
    const bool full = a.dim == (uint32_t)(kLanes * floats_per_lane(s));
    const uint32_t rows = a.negatives + 1;                  // output rows of a window
    const int kmode = rows > 2u * KC ? 3 : rows > (uint32_t)KC ? 2 : rows == (uint32_t)KC ? 1 : 0;
    for (const TrainEntry &e : kTrainTable)
        if (e.vw == s.vw && e.r == s.r && e.tail == s.tail && e.kmode == kmode) return e.get(a.window, full, update);
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

uint32_t train_lds_bytes(const KernelArgs &a, RowShape s, int update)
{
    const uint32_t rowf = kLanes * floats_per_lane(s);
    const int kmode = a.negatives + 1 > 2u * KC ? 3 : a.negatives + 1 > (uint32_t)KC ? 2 : a.negatives + 1 == (uint32_t)KC ? 1 : 0;
    const uint32_t chunk = (uint32_t)chunk_windows(floats_per_lane(s), wcap_of(a.window), update == 1);
    const uint32_t fifo = (uint32_t)fifo_entries(floats_per_lane(s), wcap_of(a.window), update == 1);
    // ring, kept-token FIFO, per-window scalars, negatives; bfloat16 storage: the rounding draws of the chunk's windows
    return (2 * a.window + 3) * rowf * 4u + fifo * 8u + chunk * 32u + chunk * a.negatives * 4u +
           (update == 2 && rounding_draws_in_lds(kmode) ? chunk * 16u : 0u);
}

hipError_t launch_init_weights(void *syn0, void *syn1neg, uint32_t vocab, uint32_t dim, uint32_t ld,
                               uint64_t seed, uint32_t storage, hipStream_t stream)
{
    const uint64_t n = (uint64_t)vocab * ld;
    const uint32_t blocks = (uint32_t)((n + 255) / 256 < 8192 ? (n + 255) / 256 : 8192);
    if (storage)
        hipLaunchKernelGGL(init_weights_bf16_kernel, dim3(blocks), dim3(256), 0, stream, static_cast<uint16_t *>(syn0),
                           static_cast<uint16_t *>(syn1neg), vocab, dim, ld, mix64(seed ^ 0x696E6974ull));
    else
        hipLaunchKernelGGL(init_weights_kernel, dim3(blocks), dim3(256), 0, stream, static_cast<float *>(syn0),
                           static_cast<float *>(syn1neg), vocab, dim, ld, mix64(seed ^ 0x696E6974ull));
    return hipGetLastError();
}

hipError_t launch_widen_rows(const void *src, float *dst, uint32_t vocab, uint32_t dim, uint32_t ld, hipStream_t stream)
{
    const uint64_t n = (uint64_t)vocab * dim;
    const uint32_t blocks = (uint32_t)((n + 255) / 256 < 8192 ? (n + 255) / 256 : 8192);
    hipLaunchKernelGGL(widen_rows_kernel, dim3(blocks), dim3(256), 0, stream, static_cast<const uint16_t *>(src), dst, vocab, dim, ld);
    return hipGetLastError();
}

hipError_t launch_reset_accum(Accum *accum, int what, hipStream_t stream)
{
    hipLaunchKernelGGL(reset_accum_kernel, dim3(1), dim3(64), 0, stream, accum, what);
    return hipGetLastError();
}

hipError_t launch_export_accum(const Accum *accum, double *loss_sum_dev, uint64_t *pairs_dev, hipStream_t stream)
{
    hipLaunchKernelGGL(export_accum_kernel, dim3(1), dim3(64), 0, stream, accum, loss_sum_dev, pairs_dev);
    return hipGetLastError();
}

hipError_t launch_plan(Accum *accum, const uint64_t *sent_off, const PlanRequest &req, hipStream_t stream)
{
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(64), 0, stream, accum, sent_off, req);
    return hipGetLastError();
}

hipError_t launch_fill_dump(const DrawDump &d, uint64_t n_tokens, uint32_t negatives, hipStream_t stream)
{
    if (n_tokens == 0) return hipSuccess;
    const uint32_t blocks = (uint32_t)((n_tokens + 255) / 256 < 16384 ? (n_tokens + 255) / 256 : 16384);
    hipLaunchKernelGGL(fill_dump_kernel, dim3(blocks), dim3(256), 0, stream, d, n_tokens, negatives);
    return hipGetLastError();
}

bool train_kernel_exists(const KernelArgs &a, int update)
{
    RowShape s;
    return pick_row_shape(a.dim, a.ld, &s) && train_fn(a, s, update) != nullptr;
}

uint32_t train_snap_floats(const KernelArgs &a)
{
    RowShape s;
    if (!pick_row_shape(a.dim, a.ld, &s) || !train_fn(a, s, 1)) return 0;
    return (2 * a.window + 2) * (uint32_t)(kLanes * floats_per_lane(s));
}

uint32_t train_resident_waves(const KernelArgs &a, int update, int device)
{
    RowShape s;
    if (!pick_row_shape(a.dim, a.ld, &s)) return 0;
    TrainFn fn = train_fn(a, s, update);
    if (!fn) return 0;
    int per_cu = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kLanes, train_lds_bytes(a, s, update)) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) return 0;
    return (uint32_t)(per_cu > 0 ? per_cu : 1) * (uint32_t)(cus > 0 ? cus : 1);
}

hipError_t launch_train(const KernelArgs &a, int update, uint32_t waves, hipStream_t stream)
{
    RowShape s;
    if (!pick_row_shape(a.dim, a.ld, &s)) return hipErrorInvalidValue;
    TrainFn fn = train_fn(a, s, update);
    if (!fn) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fn, dim3(waves), dim3(kLanes), train_lds_bytes(a, s, update), stream, a);
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
