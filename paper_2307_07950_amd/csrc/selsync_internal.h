// Internal declarations shared by the host side (context, plans, validation) and
// the device side (kernels and their launchers) of the SelSync library.  Nothing in
// here is part of the public C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace selsync {

// ---- device-visible tables --------------------------------------------------

// Pointers of one (worker k, tensor t) pair; index k*T + t.
struct TensorRec {
    const void *g;   // gradient (fp32, or bf16 in mixed mode)
    float *w;        // fp32 parameter (mixed mode: fp32 master)
    float *m;        // fp32 momentum buffer
    uint16_t *lowp;  // bf16 working copy (mixed mode only)
    float *v;        // fp32 second-moment buffer (Adam variant only, else null)
};

// One unit of work of the multi-tensor streaming kernel: `n` consecutive elements
// of one tensor of one worker, starting at element `off`.
struct ChunkRec {
    uint32_t rec;      // index into the TensorRec table
    uint32_t n_flags;  // bits 0..27: element count; bit 31: all pointers 16-byte aligned
    uint64_t off;      // first element
};

// One unit of work of the aggregation kernel: `n` consecutive elements of tensor t
// across all K replicas.
struct AggChunkRec {
    uint32_t t;
    uint32_t n_flags;
    uint64_t off;
};

// Flag bits of n_flags.  "Aligned" means: every stream of the chunk has the same phase p
// (element index mod 4 of its address relative to 16-byte alignment; bf16 streams relative to
// 8-byte alignment), so after peeling head = (4 - p) % 4 elements all streams are vector-aligned.
constexpr uint32_t kChunkAligned = 0x80000000u;
constexpr uint32_t kChunkAlignedGrads = 0x40000000u;   // aggregation chunks: gradients and momenta share the phase too
constexpr uint32_t kChunkHeadShift = 28;               // bits 28..29: head element count
constexpr uint32_t kChunkCountMask = 0x0fffffffu;

// Aggregation pointer tables (device arrays).
struct AggTables {
    float *const *w;           // [T*K]  replica parameters (mixed: masters), index t*K + k
    uint16_t *const *lowp;     // [T*K]  bf16 copies (mixed only)
    float *const *global;      // [T]
    uint16_t *const *glowp;    // [T]    (mixed only)
    const void *const *g;      // [T*K]  gradients (only when the plan has gradients)
    float *const *m;           // [T*K]  momentum buffers (only when the plan has gradients)
};

// Results of the last step plus the cumulative counters; one contiguous block so a
// blocking read is a single device-to-host copy.  Followed in memory by
//   double norm_sq[K]; double delta[K]; double smoothed[K]; int32_t flags[K];
struct DecisionHeader {
    int64_t steps_local;
    int64_t steps_sync;
    int64_t nonfinite_steps;
    double max_delta;
    int32_t sync;            // OR over the K flags of the last step
    int32_t nonfinite_now;   // some ||g||^2 of the last step was not finite
};

// Device-side state of the K significance trackers.
struct TrackerDev {
    double *hist;            // [K][window] ring buffers of raw ||g||^2
    int32_t *len;            // [K] samples stored (<= window)
    int32_t *head;           // [K] slot the next sample is written to
    double *s_prev;          // [K] previous smoothed value
    int32_t *has_prev;       // [K]
    const double *weights;   // [window] (1-alpha)^j
    double *delta_thr;       // [1] threshold delta
    DecisionHeader *out;
    double *out_norm_sq;     // [K]
    double *out_delta;       // [K]
    double *out_smoothed;    // [K]
    int32_t *out_flags;      // [K]
    int32_t K;
    int32_t window;
};

struct AdamArgs {
    float lr, b1, b2, omb1, omb2, eps, wd, gs, bc1, bc2;
    int32_t first;   // step 1: moment buffers are taken as zero
};

struct SgdArgs {
    float lr, mu, wd, gs;
    int32_t first;
};

// Launch shape for the streaming kernels.
struct LaunchCfg {
    int grid;
    int nontemporal;
    int variant = 0;   // workgroup shape of the streaming kernel
    int xcd_swizzle = 0;   // 1: XCD-aware workgroup -> chunk mapping
};

enum StreamMode { kNormOnly = 0, kUpdateOnly = 1, kUpdateAndNorm = 2 };

// ---- data partitioning (Sec. III-D), shared by the host function and the device kernel ----

// Chunk c of D samples over N workers starts here; the first D % N chunks hold one more sample.
__host__ __device__ inline int64_t chunk_start(int64_t D, int64_t N, int64_t c)
{
    const int64_t base = D / N, rem = D % N;
    return c * base + (c < rem ? c : rem);
}

// Sample index at position p of worker n's reading order.
//   scheme 0 (default partitioning): positions cover the worker's own chunk only.
//   scheme 1 (SelSync partitioning): all chunks as a circular queue rotated to chunk n,
//   i.e. chunk n, n+1, ..., N-1, 0, ..., n-1.
__host__ __device__ inline int64_t partition_index(int64_t D, int64_t N, int64_t n, int scheme, int64_t p)
{
    if (scheme == 0)
        return chunk_start(D, N, n) + p;
    // the rotated order is the tail [start(n), D) followed by the head [0, start(n))
    const int64_t tail = D - chunk_start(D, N, n);
    return p < tail ? chunk_start(D, N, n) + p : p - tail;
}

// ---- launchers (selsync_kernels.hip) --------------------------------------------

// Elements one workgroup pass of the default streaming kernel shape covers: one
// wavefront x 2 groups of 4 elements per lane (128-bit per fp32 stream, 64-bit per bf16 stream).
constexpr int kTileElems = 512;
// Chunk sizes must be a multiple of this (the smallest workgroup shape's tile).
constexpr int kChunkGranule = 256;
// Smallest aggregation tile: 256 threads x one 128-bit vector.
constexpr int kAggTileElems = 1024;

hipError_t launch_stream(StreamMode mode, bool mixed, const TensorRec *recs, const ChunkRec *chunks, int nchunks,
                         double *partials, const SgdArgs &sgd, const LaunchCfg &cfg, hipStream_t s);

// Sums partials[segs[j].x .. segs[j].y) into seg_sums[j], one workgroup per segment.
hipError_t launch_reduce(const double *partials, const int2 *segs, int nsegs, double *seg_sums, hipStream_t s);

// Adam variant of the streaming kernel: update (+ norm partials when with_norm).
hipError_t launch_stream_adam(bool with_norm, bool mixed, const TensorRec *recs, const ChunkRec *chunks, int nchunks,
                              double *partials, const AdamArgs &a, const LaunchCfg &cfg, hipStream_t s);

hipError_t launch_track(const TrackerDev &td, const double *partials, const int32_t *chunk_begin, hipStream_t s);

hipError_t launch_aggregate(bool mixed, const AggChunkRec *chunks, int nchunks, const AggTables &tabs, int K,
                            const int32_t *sync_flag, int mode, const LaunchCfg &cfg, hipStream_t s);

// out[i] = sum of partials[range_begin[i] .. range_begin[i+1]), one workgroup per range.
hipError_t launch_tensor_norms(const double *partials, const int32_t *range_begin, int nranges, double *out,
                               hipStream_t s);

// Gradient-aggregation update (Sec. III-C): when the decision is "sync" (or mode 1) every worker
// applies the mean gradient to its own parameters and momentum, otherwise its own gradient.
hipError_t launch_update_ga(bool mixed, const AggChunkRec *chunks, int nchunks, const AggTables &tabs, int K,
                            const int32_t *sync_flag, int mode, const SgdArgs &sgd, const LaunchCfg &cfg,
                            hipStream_t s);

// out[p] = partition_index(D, N, n, scheme, p) for p < count (device array).
hipError_t launch_partition_order(int64_t D, int64_t N, int64_t n, int scheme, int64_t count, int64_t *out,
                                  hipStream_t s);

hipError_t launch_reset(const TrackerDev &td, hipStream_t s);
hipError_t launch_set_delta(const TrackerDev &td, double delta, hipStream_t s);

}  // namespace selsync
