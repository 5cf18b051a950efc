// Internal declarations shared by the host API (w2v_api.hip) and the kernels (w2v_kernels.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>

#include "../../include/w2v.h"

namespace w2v {

// Device-side accumulators and the work counter, at the start of the caller's workspace.
struct Accum {
    double             loss_sum;       // sum of window losses
    unsigned long long pairs;          // (context, target) pairs trained
    unsigned long long next_sentence;  // work queue head of the current launch
    unsigned long long dropped;        // tokens with ids outside [0, V)
    unsigned long long kept;           // tokens that survived subsampling (windows processed)
    // Work plan of the current launch, written by the planning kernel that precedes it: the first coarse_sent
    // sentences are handed out as 2^unit_shift units each, the others as 2^fine_shift, n_units in all.
    unsigned long long coarse_sent, n_units;
    uint32_t           unit_shift, fine_shift;
};

// How a launch's sentences are to be cut into units of work (input of the planning kernel).
struct PlanRequest {
    uint64_t n_sent;
    uint64_t waves;               // wavefronts the launch will have
    int32_t  forced_unit_shift;   // -1: choose from the sizes
    int32_t  forced_fine_shift;   // -1: choose
    uint64_t forced_coarse_sent;  // used with forced_fine_shift
};

// Optional dump of the window kernel's own integer decisions (all NULL in production), indexed by token offset in
// `tokens`: keep[t] = 1 and width[t], neg[t*N + k] for every token that gets a window in the launch.
struct DrawDump {
    uint8_t *keep, *width;
    int32_t *neg;
};

// Layout of the caller-provided workspace (all offsets multiples of 256 bytes).
struct WorkspaceLayout {
    uint64_t accum_off, thr_off, snap_off, table_off, total;
};
WorkspaceLayout workspace_layout(uint32_t vocab, uint32_t table_size, uint64_t snap_bytes);
// most wavefronts a launch with summed updates uses (each owns a snapshot area in the workspace)
constexpr uint32_t kMaxSummedWaves = 4096;

// Everything a training / draw kernel needs; passed by value.
struct KernelArgs {
    float             *syn0, *syn1neg;
    const int32_t     *tokens;
    const uint64_t    *sent_off;
    const int32_t     *table;
    const uint32_t    *thr;
    Accum             *accum;
    uint64_t           n_sent, first_pos, key;
    uint64_t           lr_done_base;   // epoch * tokens_per_epoch
    uint64_t           lr_all;         // total_epochs * tokens_per_epoch
    double             lr0, lr_min_frac;
    uint32_t           vocab, dim, ld, window, negatives, window_mode, table_size;
    uint32_t           subsample;      // 0: every threshold is "always keep", thr is not read
    uint32_t           neg_shift;      // 0: negatives drawn at each window's own position; s: at the first position
                                       // of the stretch of 2^s tokens (offsets in the sentence) the centre lies in
    // Summed lock-free updates (window kernel instantiated with SUMMED): wavefront w keeps the value each of its
    // ring slots had when it was fetched in snap + w * snap_stride floats.
    float             *snap;
    uint32_t           snap_stride;
    DrawDump           dump;
};

using TrainFn = void (*)(KernelArgs);

// How a row of `dim` floats is spread over the 64 lanes of a wavefront: R chunks of VW
// consecutive floats per lane, chunk r of lane l starting at float (r*64 + l)*VW, then `tail`
// chunks of one float each (chunk t of lane l is float 64*VW*R + t*64 + l).
struct RowShape { int vw, r, tail; };
inline int floats_per_lane(RowShape s) { return s.vw * s.r + s.tail; }
bool pick_row_shape(uint32_t dim, uint32_t ld, RowShape *out);

// LDS bytes one wavefront (= one workgroup) of the window kernel needs.
uint32_t train_lds_bytes(const KernelArgs &a, RowShape s, int update);

// Launchers (all asynchronous on `stream`).  Return hipSuccess or the launch error.
hipError_t launch_init_weights(void *syn0, void *syn1neg, uint32_t vocab, uint32_t dim, uint32_t ld,
                               uint64_t seed, uint32_t storage, hipStream_t stream);
// dense float copy of a bfloat16 table: dst[i*dim + j] = widen(src[i*ld + j]); dst is device memory
hipError_t launch_widen_rows(const void *src, float *dst, uint32_t vocab, uint32_t dim, uint32_t ld, hipStream_t stream);
hipError_t launch_reset_accum(Accum *accum, int what /*1: work counter only, 2: everything*/, hipStream_t stream);
// resets the work counter and writes the launch's work plan into accum (the token count of the call is read from
// sent_off on the device)
hipError_t launch_plan(Accum *accum, const uint64_t *sent_off, const PlanRequest &req, hipStream_t stream);
hipError_t launch_train(const KernelArgs &a, int update, uint32_t waves, hipStream_t stream);
// is there an instantiation of the window kernel for this shape and update mode (0 overwrite, 1 summed, 2 bfloat16)?
bool train_kernel_exists(const KernelArgs &a, int update);
// floats of snapshot space one wavefront of the summed mode needs (0 if the shape has no such instantiation)
uint32_t train_snap_floats(const KernelArgs &a);
hipError_t launch_fill_dump(const DrawDump &d, uint64_t n_tokens, uint32_t negatives, hipStream_t stream);
hipError_t launch_train_naive(const KernelArgs &a, uint32_t waves, hipStream_t stream);
hipError_t launch_draws(const KernelArgs &a, uint64_t n_tokens_hint, uint8_t *keep, uint8_t *width, int32_t *neg,
                        hipStream_t stream);
hipError_t launch_reduce_selftest(const float *in, float *out, hipStream_t stream);
// The library's own scratch memory for w2v_train_epoch_static: a file-scope device array of kStaticScratchBytes, one
// copy per GPU.  static_scratch() returns its device address on `device`, which must be the current device (asked of
// the runtime once per device).
constexpr uint64_t kStaticScratchBytes = 32ull << 20;
hipError_t static_scratch(int device, unsigned char **ptr);
// copies the loss sum and the pair count of an accumulator block to device locations of the caller (either may be NULL)
hipError_t launch_export_accum(const Accum *accum, double *loss_sum_dev, uint64_t *pairs_dev, hipStream_t stream);
// waves that fit the device at once for this configuration (0 on error)
uint32_t train_resident_waves(const KernelArgs &a, int update, int device);
uint32_t naive_resident_waves(int device);

}  // namespace w2v

struct w2v_ctx {
    w2v_config           cfg;
    w2v::WorkspaceLayout ws;
    uint32_t             table_size = 0;
    bool                 table_built = false;
    int                  forced_unit_shift = -1;   // test override of the work-queue granularity (-1: automatic)
    int                  forced_fine_shift = -1;   // test override of the granularity of the queue's end (-1: automatic)
    uint64_t             forced_coarse_sent = 0;   // ... and of the sentence it begins with
    std::string          err;
    // host-fed training (created on first use): copy stream, and per staging half an event for "filled"
    // (recorded on the copy stream) and one for "trained, may be refilled" (recorded on the caller's stream)
    hipStream_t          copy_stream = nullptr;
    hipEvent_t           filled[2] = {nullptr, nullptr};
    hipEvent_t           drained[2] = {nullptr, nullptr};
    bool                 drained_recorded[2] = {false, false};
    double               kept_fraction = 1.0;  // expected share of the tokens that survive subsampling (from the counts)
    uint64_t             resident_waves[3] = {0, 0, 0}; // wavefronts of the window kernel the device holds, by update mode (0: not asked yet)
    uint32_t             snap_floats = 0;    // snapshot floats per wavefront of the summed mode (0: no such kernel for this shape)
    bool                 flat_corpus = false; // from the counts: the rows one L2 holds carry a small share of the tokens
    int                  forced_update = -1; // test override: update mode of every launch, strict order included (-1: by the rules)
    double               collision_mass = 0.0; // sum over words of (share of the kept tokens)^2, from the counts
    int                  last_update = 0;    // update mode and wavefronts of the last launch (test surface)
    uint64_t             last_waves = 0;
    int                  next_half = 0;      // staging half the next batch goes to (alternates across calls too)
};
