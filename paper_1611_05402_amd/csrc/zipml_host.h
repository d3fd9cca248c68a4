// Host-side helpers shared by the libzipml entry points.
#pragma once
#include <hip/hip_runtime.h>
#include <atomic>
#include <stddef.h>
#include <stdio.h>
#include <stdint.h>

#include "../../include/zipml.h"

namespace zipml {

inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool valid_bits(int bits) { return bits >= 1 && bits <= 8; }

// Packed layout (private).  A unit is 32 codes of `bits` bits: a little-endian bit string of
// `bits` dwords, stored contiguously so that a thread fetches its unit with the widest loads its
// alignment allows.  n is padded to a multiple of 64, d to a multiple of 32.
//   copy 2 (dot pass):      unit = one sample x 32 features
//                           [feature group g][sample i][bits dwords]
//   copy 1 (gradient pass): unit = one feature x 32 samples
//                           [feature group g][group of 32 samples][feature in group][bits dwords]
struct Layout {
    int64_t n, d, n_pad, d_pad;
    int64_t d32;    // feature groups
    int64_t n32;    // sample groups of 32 (copy 1)
    int64_t nb64;   // sample blocks of 64 (copy 2)
    int bits;
    size_t bytes() const { return (size_t)n_pad * (size_t)d_pad * (size_t)bits / 8; }
};
inline Layout make_layout(int64_t n, int64_t d, int bits)
{
    Layout L;
    L.n = n; L.d = d; L.bits = bits;
    L.n_pad = round_up(n, 64); L.d_pad = round_up(d, 32);
    L.d32 = L.d_pad / 32; L.n32 = L.n_pad / 32; L.nb64 = L.n_pad / 64;
    return L;
}

// Workspace carving (all offsets 256-byte aligned).
struct Workspace {
    static constexpr size_t kStatus = 0;          // int32 status word + counters   (4 KiB)
    static constexpr size_t kSync = 4096;         // grid barrier counter                  (256 B)
    static constexpr size_t kBound = 4096 + 256;  // magnitude bounds of the dot exchange: 4 doubles
    static constexpr size_t kEven = 4096 + 1024;  // kEvenBlocks ints: levels evenly spaced, per block of features
    // (64, not more: with 128 or 256 blocks in the preparation launch the epoch kernel that
    // follows it ran 3 % slower at batch 256, measured)
    static constexpr int kEvenBlocks = 64;
    static constexpr size_t kNorm = 8192;         // norm exchange: 2 x 3 x 512 doubles (24 KiB)
    static constexpr size_t kAcc = 8192 + 24576;  // exchange buffers, 64-bit words (see below)
    static constexpr int kAccBuffers = 4;
    // One set of exchange buffers: kAccBuffers x acc_words(batch of one exchange), with room for
    // the sums of both code pairs of the symmetrised estimator and the side words.
    static size_t acc_words(int64_t batch) { return (size_t)round_up(2 * batch + 64, 64); }
    // A large minibatch is split over up to kMaxReplicas sets of workgroups; every replica has its
    // own set of exchange buffers for its share of the minibatch (R * acc_words(batch / R) <=
    // 2 * batch + 64 * R words per buffer), and the replicas exchange gradients through two
    // buffers of kGradWords tagged words (at most 256 workgroups x 128 features), which follow
    // the exchange buffers in use.
    static constexpr int kMaxReplicas = 256;
    static constexpr size_t kGradWords = 256 * 128;
    static size_t sgd_bytes(int64_t batch)
    {
        return kAcc + (kAccBuffers * (2 * (size_t)round_up(batch, 64) + 64 * kMaxReplicas) + 2 * kGradWords) * 8;
    }
    // Very large minibatches (kRowsMinBatch samples or more, a multiple of 64) may take the
    // sample-owner kernel: per-feature constants (2 arrays), one gradient per workgroup (at most
    // kMaxRowsWgs) and one sum of residuals per workgroup, all fp32, behind everything else.
    static constexpr int64_t kRowsMinBatch = 16384;
    static constexpr int kMaxRowsWgs = 256;
    static size_t rows_bytes(int64_t d, int64_t batch)
    {
        if (batch < kRowsMinBatch || batch % 64 != 0) return 0;
        return ((size_t)(kMaxRowsWgs + 2) * (size_t)round_up(d, 64) + kMaxRowsWgs + 64) * 4;
    }
    // Exchange through tagged stores (zipml_sgd_mfma.h): two buffers of one row of exchange words
    // per workgroup (at most 256, and no more than there are groups of 32 features) plus one row
    // of results; a row holds the sums of both code pairs of one exchange (at most 2048 samples)
    // and two side words, rounded up to pieces of eight.  Behind everything else, 256-byte aligned.
    static size_t xchg_row_words(int64_t batch)
    {
        return (size_t)round_up(2 * (batch < 2048 ? batch : 2048) + 2, 8);
    }
    static size_t xchg_bytes(int64_t d, int64_t batch)
    {
        const int64_t d32 = round_up(d, 32) / 32;
        const size_t wmax = (size_t)(d32 < 256 ? d32 : 256);
        return 2 * (wmax + 1) * xchg_row_words(batch) * 8;
    }
    static size_t xchg_offset(int64_t d, int64_t batch)
    {
        return (size_t)round_up((int64_t)(sgd_bytes(batch) + (size_t)round_up(d, 64) * 4 + rows_bytes(d, batch)), 256);
    }
};

// Development knobs (zipml_debug_set): process-wide overrides of choices the library otherwise
// makes by itself, used by sweeps and by tests that steer kernel selection.  -1 = automatic.
// The library never reads the environment.
constexpr int kKnobs = ZIPML_KNOB_COUNT;
inline std::atomic<long long> g_knob[kKnobs] = {};   // value + 1, so that zero-initialised means "automatic"
inline long long knob(int k) { return g_knob[k].load(std::memory_order_relaxed) - 1; }

// Called on entry of every API function: hipGetLastError() is sticky per host thread, so an
// error left behind by an earlier, unrelated runtime call of the caller (e.g. a pointer query on
// host memory) must not be mistaken for a failed launch of ours.
inline hipStream_t entry_stream(void *stream)
{
    (void)hipGetLastError();
    return (hipStream_t)stream;
}

// Maps a HIP status to a library status; the HIP error text goes to stderr so that ZIPML_ELAUNCH
// can be diagnosed.
inline int hip_check_at(hipError_t e, const char *file, int line)
{
    if (e == hipSuccess) return ZIPML_OK;
    fprintf(stderr, "libzipml: HIP error '%s' at %s:%d\n", hipGetErrorString(e), file, line);
    return ZIPML_ELAUNCH;
}
#define hip_check(e) hip_check_at((e), __FILE__, __LINE__)
#define HIP_FAILED(e) (hip_check_at((e), __FILE__, __LINE__) != ZIPML_OK)

}  // namespace zipml
