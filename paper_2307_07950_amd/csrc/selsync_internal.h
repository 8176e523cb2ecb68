// Internal declarations shared by the host side (context, plans, validation) and
// the device side (kernels and their launchers) of the SelSync library.  Nothing in
// here is part of the public C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace selsync {

// ---- device-visible tables --------------------------------------------------

// One (worker k, tensor t) pair; index k*T + t.  64 bytes, so a record never straddles a
// cache line and one scalar load fetches it.
struct alignas(64) TensorRec {
    const void *g;   // gradient (fp32, or bf16 in mixed mode)
    float *w;        // fp32 parameter (mixed mode: fp32 master)
    float *m;        // fp32 momentum buffer
    uint16_t *lowp;  // bf16 working copy (mixed mode only)
    float *v;        // fp32 second-moment buffer (Adam variant only, else null)
    int64_t numel;   // elements of the tensor
    uint32_t flags;  // kChunkAligned | head bits (same meaning as in AggChunkRec::n_flags)
    uint32_t lead;   // elements between the last chunk-size-aligned address and the first element
};

// One unit of work of the multi-tensor streaming kernel: piece j of one tensor of one
// worker, i.e. elements [j*chunk_elems - lead, (j+1)*chunk_elems - lead) clipped to
// [0, numel): pieces are cut where the tensor's addresses cross multiples of the chunk
// size.  8 bytes: at 256 elements per chunk the table is 1/128 of one fp32 stream.
struct ChunkRec {
    uint32_t rec;   // index into the TensorRec table; kNoChunk marks a padding slot
    uint32_t j;     // chunk index inside the tensor
};
constexpr uint32_t kNoChunk = 0xffffffffu;

// Where chunk c's table record and partial sum live.  Workgroups of a launch go to the 8
// XCDs (each with its own L2) round-robin by workgroup id.  The slots are stored as 8 stripes
// of `per` slots and workgroup b works on stripe b % 8, so the records and partial sums of
// one XCD's workgroups are contiguous in memory: every table line is fetched by one L2
// instead of eight, every line of partial sums is written by one, while chunks are still
// dispatched in model order: chunk c sits in slot (c%8)*per + c/8.  (per = 0: plain index,
// used for arrays that are not striped, such as the per-segment sums.)
__host__ __device__ inline int64_t chunk_slot(int64_t c, int per)
{
    return per > 0 ? (c & 7) * (int64_t)per + (c >> 3) : c;
}

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
constexpr uint32_t kChunkAlignedGrads = 0x40000000u;   // aggregation chunks: gradients (and momenta, if bound) share the phase too
constexpr uint32_t kChunkHeadShift = 28;               // bits 28..29: head element count
constexpr uint32_t kChunkCountMask = 0x0fffffffu;

// Aggregation pointer tables (device arrays).
struct AggTables {
    float *const *w;           // [T*K]  replica parameters (mixed: masters), index t*K + k
    uint16_t *const *lowp;     // [T*K]  bf16 copies (mixed only)
    float *const *global;      // [T]
    uint16_t *const *glowp;    // [T]    (mixed only)
    const void *const *g;      // [T*K]  gradients (only when the plan has gradients)
    float *const *m;           // [T*K]  momentum buffers (only when the plan has them)
    float *const *v;           // [T*K]  second-moment buffers (filled when they are bound)
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
    int32_t nesterov;
};

// Workgroup shape of the K-way kernels.
//   kAggCoarse: 256 threads, 4 vectors of 4 elements per lane and replica (made for 4096-element pieces):
//               few workgroups, so a launch that only reads the decision and exits is cheap;
//   kAggFine:   one wavefront, one vector per lane and replica (made for 256-element pieces): the
//               shape with the highest bandwidth when the launch does work.
enum AggShape { kAggCoarse = 0, kAggFine = 1 };

// One table of the K-way kernels.  per8 > 0: 8 stripes of per8 records, piece p in slot
// (p % 8) * per8 + p / 8 (padding records hold n = 0) and nslots = 8 * per8; per8 = 0: plain.
struct AggTable {
    const AggChunkRec *recs = nullptr;
    int nslots = 0;            // grid size of a launch over the table
    int per8 = 0;
    AggShape shape = kAggCoarse;
};

// Geometry of a plan's chunk table (see chunk_slot).
struct StreamTable {
    const TensorRec *recs = nullptr;
    const ChunkRec *slots = nullptr;
    double *partials = nullptr;    // one per slot
    int nchunks = 0;               // real chunks
    int nslots = 0;                // table entries including padding: 8 * per
    int per = 0;                   // slots per stripe
    uint32_t chunk_elems = 0;
    bool has_momentum = true;      // false: momentum-free plan (no m buffers bound)
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

// Chunk sizes are a multiple of this: one wavefront x one group of 4 elements per lane
// (128 bits per fp32 stream, 64 bits per bf16 stream).
constexpr int kChunkGranule = 256;
// Stripes are padded to a multiple of this many slots (a multiple of every chunks-per-wave count).
constexpr int kStripeGranule = 16;
// Smallest aggregation tile: 256 threads x one 128-bit vector.
constexpr int kAggTileElems = 1024;

// With `pred` the launch only works while *pred == pred_want (device-side word), else it exits.
hipError_t launch_stream(StreamMode mode, bool mixed, const StreamTable &tab, const SgdArgs &sgd, bool nontemporal,
                         hipStream_t s, const int32_t *pred = nullptr, int pred_want = 0);

// Adam variant of the streaming kernel: update (+ norm partials when with_norm).
hipError_t launch_stream_adam(bool with_norm, bool mixed, const StreamTable &tab, const AdamArgs &a, bool nontemporal,
                              hipStream_t s, const int32_t *pred = nullptr, int pred_want = 0);

// Sums the partials of chunks segs[j].x .. segs[j].y - 1 into seg_sums[j], one workgroup per
// segment.  slot_per: see chunk_slot().
hipError_t launch_reduce(const double *partials, int slot_per, const int2 *segs, int nsegs, double *seg_sums,
                         hipStream_t s);

// values[begin[k] .. begin[k+1]) are worker k's partial sums: per-chunk ones (looked up through
// chunk_slot(., slot_per)) or per-segment ones (slot_per = 0).
hipError_t launch_track(const TrackerDev &td, const double *values, int slot_per, const int32_t *begin, hipStream_t s);

hipError_t launch_aggregate(bool mixed, const AggTable &t, const AggTables &tabs, int K, const int32_t *sync_flag,
                            int mode, bool nontemporal, hipStream_t s);

// out[i] = sum of the partials of chunks range_begin[i] .. range_begin[i+1] - 1, one workgroup per range.
hipError_t launch_tensor_norms(const double *partials, int slot_per, const int32_t *range_begin, int nranges,
                               double *out, hipStream_t s);

// What a launch of the gradient-aggregation update does with the device-side decision.
enum GaMode { kGaSyncOnly = 0, kGaAlways = 1, kGaSyncOrLocal = 2 };

// Update of gradient aggregation (Sec. III-C): on "sync" (or kGaAlways) every worker applies the
// mean gradient to its own parameters and optimiser state; on "local" the launch exits
// (kGaSyncOnly: the caller runs the plain local update in a launch of its own) or applies every
// worker's own gradient itself (kGaSyncOrLocal).
hipError_t launch_update_ga(bool mixed, bool has_momentum, const AggTable &t, const AggTables &tabs, int K,
                            const int32_t *sync_flag, int mode, const SgdArgs &sgd, bool nontemporal, hipStream_t s);
// ... with Adam as the update (first and second moment buffers per worker).
hipError_t launch_update_ga_adam(bool mixed, const AggTable &t, const AggTables &tabs, int K, const int32_t *sync_flag,
                                 int mode, const AdamArgs &a, bool nontemporal, hipStream_t s);

// One whole synchronous iteration in one pass over the striped table of 256-element pieces: per-worker
// squared-gradient partials (worker k's piece p is "chunk" k * nslots + p of a partial array striped with
// per = K * per8, see chunk_slot), local update, mean of the updated parameters into every replica and the
// global model.
hipError_t launch_sync_step(bool mixed, bool has_momentum, const AggTable &t, const AggTables &tabs, int K,
                            const SgdArgs &sgd, double *partials, bool nontemporal, hipStream_t s);
// ... with Adam as the update (second-moment buffers bound).
hipError_t launch_sync_step_adam(bool mixed, const AggTable &t, const AggTables &tabs, int K, const AdamArgs &a,
                                 double *partials, bool nontemporal, hipStream_t s);

// out[p] = partition_index(D, N, n, scheme, p) for p < count (device array).
hipError_t launch_partition_order(int64_t D, int64_t N, int64_t n, int scheme, int64_t count, int64_t *out,
                                  hipStream_t s);

hipError_t launch_reset(const TrackerDev &td, hipStream_t s);
hipError_t launch_set_delta(const TrackerDev &td, double delta, hipStream_t s);

}  // namespace selsync
