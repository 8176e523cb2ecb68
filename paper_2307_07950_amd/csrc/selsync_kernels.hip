// CDNA4 (gfx950) kernels of the SelSync per-step path and their launchers.
//
//   k_stream     multi-tensor-apply over a chunk table: fused local SGD update
//                (Alg. 1 line 9) and/or per-chunk sum of squared gradients
//                (the ||g_i||^2 of Alg. 1 line 8).  One read of g serves both.
//   k_track      deterministic final pass over the per-chunk partials, then the
//                windowed EWMA, Eq. 2, the delta rule and the any-worker OR
//                (Sec. III-A/B, Alg. 1 lines 8, 10-13), all K workers in one block.
//   k_aggregate  K-way replica mean written to the global model and back to every
//                replica (Alg. 1 lines 14-15), predicated on the device-side decision.
//
// All three are HBM-bandwidth bound (<= 0.4 flop/byte), so there is no MFMA use:
// the design is 128-bit coalesced non-temporal accesses, one-shot grids of single-wave
// workgroups that each carry as little work as one vector per lane and stream (the
// hardware dispatcher then streams through the model in order, one retired wave at a
// time), tables laid out per XCD, and no atomics (every partial has a fixed slot and
// every sum a fixed order, so results are run-to-run identical for tensors at the same
// addresses modulo the chunk size -- the cutting of tensors into pieces follows addresses).
//
// fp32 arithmetic of the update is written to round once per operation; the file
// is compiled with -ffp-contract=off and the pragma below so no multiply-add is fused.
#include "selsync_internal.h"

#pragma clang fp contract(off)

namespace selsync {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Tensor pointers come out of tables in memory, so the compiler only knows them as
// generic (flat) addresses.  They are device-memory addresses by construction (checked
// at plan time); casting them to the global address space yields global_load/global_store
// instead of the slower flat forms.
#define SELSYNC_GLOBAL __attribute__((address_space(1)))

template <typename T>
__device__ __forceinline__ SELSYNC_GLOBAL T *as_global(const void *p)
{
    return (SELSYNC_GLOBAL T *)(p);
}

template <bool NT, typename T>
__device__ __forceinline__ T ld(const SELSYNC_GLOBAL T *p)
{
    if (NT)
        return __builtin_nontemporal_load(p);
    return *p;
}

template <bool NT, typename T>
__device__ __forceinline__ void st(SELSYNC_GLOBAL T *p, T v)
{
    if (NT)
        __builtin_nontemporal_store(v, p);
    else
        *p = v;
}

// bf16 <-> fp32.  Widening is exact; narrowing rounds to nearest, ties to even, and
// keeps NaN a quiet NaN.
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ __forceinline__ uint32_t bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t bf16_pack(float lo, float hi) { return bf16_bits(lo) | (bf16_bits(hi) << 16); }
// Four bf16 values in two dwords -> four fp32 values (exact).
__device__ __forceinline__ f32x4 widen4(u32x2 v)
{
    f32x4 g;
    g.x = bf16_lo(v.x);
    g.y = bf16_hi(v.x);
    g.z = bf16_lo(v.y);
    g.w = bf16_hi(v.y);
    return g;
}

// Elements to process one by one before the 16-byte aligned body of a chunk starts (0..3).
__device__ __forceinline__ uint32_t chunk_head(uint32_t n_flags, uint32_t n)
{
    const uint32_t h = (n_flags >> kChunkHeadShift) & 3u;
    return h < n ? h : n;
}

// Sum over the 64 lanes of a wavefront in a fixed butterfly order; result in lane 0.
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        v += __shfl_down(v, o, 64);
    return v;
}

// Sum over the 64 lanes with data-parallel-primitive moves (no LDS crossbar traffic, a few
// cycles per step); result in lane 63.  Fixed order: inclusive scan inside each row of 16
// lanes (shifts by 1, 2, 4, 8), then row 0's total is added to row 1 and row 2's to row 3,
// then the total of rows 0-1 to rows 2-3.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_add(double v)
{
    // lanes without a valid source (or masked out) receive the `old` operand, 0, i.e. add +0.0
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, ROW_MASK, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, ROW_MASK, 0xf, false);
    return v + __hiloint2double(hi, lo);
}

__device__ __forceinline__ double wave_sum_to_last_lane(double v)
{
    v = dpp_add<0x111, 0xf>(v);   // row_shr:1
    v = dpp_add<0x112, 0xf>(v);   // row_shr:2
    v = dpp_add<0x114, 0xf>(v);   // row_shr:4
    v = dpp_add<0x118, 0xf>(v);   // row_shr:8
    v = dpp_add<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
    v = dpp_add<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3
    return v;
}

// ---------------------------------------------------------------- optimiser policies

// Local SGD with momentum and weight decay (Alg. 1 line 9), one rounding per operation:
//   gh = fl(gs*g); x += gh^2 in fp64 (the product of two fp32 values is exact in fp64);
//   d = fl(gh + fl(wd*w)); m = first ? d : fl(fl(mu*m) + d); w = fl(w - fl(lr*m)).
// Nesterov form: the step direction is fl(d + fl(mu*m)) with the new m instead of m.
struct SgdOpt {
    typedef SgdArgs Args;
    static constexpr bool kMomentum = true;
    static constexpr bool kSecondMoment = false;
    template <bool UPD, bool NORM>
    static __device__ __forceinline__ void elem(float g, float &w, float &m, float &, const Args &a, double &acc)
    {
        const float gh = a.gs * g;
        if (NORM)
            acc = __builtin_fma((double)gh, (double)gh, acc);
        if (UPD) {
            const float dec = a.wd * w;
            const float d = gh + dec;
            float mom = d;
            if (!a.first) {
                const float mm = a.mu * m;
                mom = mm + d;
            }
            float dir = mom;
            if (a.nesterov) {
                const float look = a.mu * mom;
                dir = d + look;
            }
            const float stepv = a.lr * dir;
            m = mom;
            w = w - stepv;
        }
    }
};

// Momentum-free SGD (the Transformer recipe of Sec. IV-A): no buffer is read or written,
//   gh = fl(gs*g); d = fl(gh + fl(wd*w)); w = fl(w - fl(lr*d)).
struct PlainSgdOpt {
    typedef SgdArgs Args;
    static constexpr bool kMomentum = false;
    static constexpr bool kSecondMoment = false;
    template <bool UPD, bool NORM>
    static __device__ __forceinline__ void elem(float g, float &w, float &, float &, const Args &a, double &acc)
    {
        const float gh = a.gs * g;
        if (NORM)
            acc = __builtin_fma((double)gh, (double)gh, acc);
        if (UPD) {
            const float dec = a.wd * w;
            const float d = gh + dec;
            const float stepv = a.lr * d;
            w = w - stepv;
        }
    }
};

// Adam (optimiser of the AlexNet recipe, Sec. IV-A), fp32, one rounding per operation;
// division and square root are the correctly rounded ones:
//   gh = gs*g; gd = gh + wd*w; m = b1*m + omb1*gd; v = b2*v + (omb2*gd)*gd;
//   w = w - (lr*(m/bc1)) / (sqrt(v/bc2) + eps)
// On the first step the moment buffers are not read (taken as zero).
struct AdamOpt {
    typedef AdamArgs Args;
    static constexpr bool kMomentum = true;
    static constexpr bool kSecondMoment = true;
    template <bool UPD, bool NORM>
    static __device__ __forceinline__ void elem(float g, float &w, float &m, float &v, const Args &a, double &acc)
    {
        const float gh = a.gs * g;
        if (NORM)
            acc = __builtin_fma((double)gh, (double)gh, acc);
        const float dec = a.wd * w;
        const float gd = gh + dec;
        const float t1 = a.b1 * m;
        const float t2 = a.omb1 * gd;
        const float mn = t1 + t2;
        const float t3 = a.b2 * v;
        const float t4 = a.omb2 * gd;
        const float t5 = t4 * gd;
        const float vn = t3 + t5;
        const float mh = mn / a.bc1;
        const float vh = vn / a.bc2;
        const float num = a.lr * mh;
        const float den = __builtin_sqrtf(vh) + a.eps;
        const float q = num / den;
        m = mn;
        v = vn;
        w = w - q;
    }
};

// Four consecutive elements held in 128-bit registers.
template <class OPT, bool UPD, bool NORM>
__device__ __forceinline__ void elem4(const f32x4 &g, f32x4 &w, f32x4 &m, f32x4 &v, const typename OPT::Args &a,
                                      double &acc)
{
    float w0 = w.x, w1 = w.y, w2 = w.z, w3 = w.w;
    float m0 = m.x, m1 = m.y, m2 = m.z, m3 = m.w;
    float v0 = v.x, v1 = v.y, v2 = v.z, v3 = v.w;
    OPT::template elem<UPD, NORM>(g.x, w0, m0, v0, a, acc);
    OPT::template elem<UPD, NORM>(g.y, w1, m1, v1, a, acc);
    OPT::template elem<UPD, NORM>(g.z, w2, m2, v2, a, acc);
    OPT::template elem<UPD, NORM>(g.w, w3, m3, v3, a, acc);
    w.x = w0; w.y = w1; w.z = w2; w.w = w3;
    m.x = m0; m.y = m1; m.z = m2; m.w = m3;
    v.x = v0; v.y = v1; v.z = v2; v.w = v3;
}

// ---------------------------------------------------------------- k_stream

// What a wavefront knows about one chunk (all of it wave-uniform, i.e. in scalar registers).
// An aligned chunk is `head` single elements, `nvec` groups of 4 elements starting at element
// off + head (every stream vector-aligned there), and a ragged tail; an unaligned one has
// nvec = 0 and is walked element by element.  n = 0 marks a padding slot.
struct Chunk {
    TensorRec r;
    uint64_t off;
    uint32_t n, head, nvec;
};

__device__ __forceinline__ Chunk lookup_chunk(const TensorRec *__restrict__ recs, const ChunkRec *__restrict__ slots,
                                              int slot, int nslots, uint32_t chunk_elems)
{
    Chunk ck;
    ChunkRec cr;
    cr.rec = kNoChunk;
    cr.j = 0;
    if (slot < nslots)
        cr = slots[slot];
    const bool real = cr.rec != kNoChunk;
    ck.r = recs[real ? cr.rec : 0u];
    // piece j in "virtual" element indices (lead + element): [j*chunk, (j+1)*chunk) clipped to
    // [lead, lead + numel)
    const uint64_t lead = ck.r.lead;
    const uint64_t vb = (uint64_t)cr.j * chunk_elems;
    const uint64_t vlast = lead + (uint64_t)ck.r.numel;
    const uint64_t ve = vb + chunk_elems < vlast ? vb + chunk_elems : vlast;
    ck.off = vb > lead ? vb - lead : 0u;
    ck.n = real ? (uint32_t)(ve - lead - ck.off) : 0u;
    ck.head = 0;
    ck.nvec = 0;
    if (ck.r.flags & kChunkAligned) {
        // only the first piece can start off vector alignment; later ones start on a
        // chunk-size-aligned address
        const uint32_t h = cr.j == 0 ? (ck.r.flags >> kChunkHeadShift) & 3u : 0u;
        ck.head = h < ck.n ? h : ck.n;
        ck.nvec = (ck.n - ck.head) / 4;
    }
    return ck;
}

// 128-bit registers of one tile: one group of 4 elements per lane and stream.
struct TileRegs {
    f32x4 g, w, m, v;
};

// Issue the loads of tile [base, base + 64) of the chunk's vector body.  Every stream is read
// with consecutive lanes on consecutive addresses (bf16 gradients: 8 bytes per lane).
template <class OPT, bool MIXED, bool UPD, bool NT>
__device__ __forceinline__ void load_tile(const Chunk &ck, uint32_t base, uint32_t tid, int first, TileRegs &t)
{
    const uint64_t e0 = ck.off + ck.head;
    const SELSYNC_GLOBAL f32x4 *g4 = as_global<const f32x4>(reinterpret_cast<const float *>(ck.r.g) + e0);
    const SELSYNC_GLOBAL u32x2 *gb4 = as_global<const u32x2>(reinterpret_cast<const uint16_t *>(ck.r.g) + e0);
    const SELSYNC_GLOBAL f32x4 *w4 = as_global<const f32x4>(ck.r.w + e0);
    const SELSYNC_GLOBAL f32x4 *m4 = as_global<const f32x4>(ck.r.m + e0);
    const SELSYNC_GLOBAL f32x4 *v4 = as_global<const f32x4>(ck.r.v + e0);
    const uint32_t i = base + tid;
    t.g = 0.f;
    t.w = 0.f;
    t.m = 0.f;
    t.v = 0.f;
    if (i < ck.nvec) {
        if (MIXED)
            t.g = widen4(ld<NT>(gb4 + i));
        else
            t.g = ld<NT>(g4 + i);
        if (UPD) {
            t.w = ld<NT>(w4 + i);
            if (OPT::kMomentum && !first) {
                t.m = ld<NT>(m4 + i);
                if (OPT::kSecondMoment)
                    t.v = ld<NT>(v4 + i);
            }
        }
    }
}

// Arithmetic and stores of the tile loaded by load_tile.
template <class OPT, bool MIXED, bool UPD, bool NORM, bool NT>
__device__ __forceinline__ void finish_tile(const Chunk &ck, uint32_t base, uint32_t tid, const typename OPT::Args &a,
                                            TileRegs &t, double &acc)
{
    const uint64_t e0 = ck.off + ck.head;
    SELSYNC_GLOBAL f32x4 *w4 = as_global<f32x4>(ck.r.w + e0);
    SELSYNC_GLOBAL f32x4 *m4 = as_global<f32x4>(ck.r.m + e0);
    SELSYNC_GLOBAL f32x4 *v4 = as_global<f32x4>(ck.r.v + e0);
    SELSYNC_GLOBAL u32x2 *c4 = as_global<u32x2>(ck.r.lowp + e0);
    const uint32_t i = base + tid;
    if (i < ck.nvec) {
        elem4<OPT, UPD, NORM>(t.g, t.w, t.m, t.v, a, acc);
        if (UPD) {
            st<NT>(w4 + i, t.w);
            if (OPT::kMomentum)
                st<NT>(m4 + i, t.m);
            if (OPT::kSecondMoment)
                st<NT>(v4 + i, t.v);
            if (MIXED) {
                u32x2 cv;
                cv.x = bf16_pack(t.w.x, t.w.y);
                cv.y = bf16_pack(t.w.z, t.w.w);
                st<NT>(c4 + i, cv);
            }
        }
    }
}

// Elements [begin, end) of a chunk one at a time (peeled head, ragged tail, or all of an
// unaligned chunk).  Still coalesced: lane i takes element begin + i.
template <class OPT, bool MIXED, bool UPD, bool NORM>
__device__ __forceinline__ void scalar_range(const Chunk &ck, uint32_t begin, uint32_t end, uint32_t tid,
                                             const typename OPT::Args &a, double &acc)
{
    const SELSYNC_GLOBAL float *gf = as_global<const float>(ck.r.g);
    const SELSYNC_GLOBAL uint16_t *gh = as_global<const uint16_t>(ck.r.g);
    SELSYNC_GLOBAL float *wp = as_global<float>(ck.r.w);
    SELSYNC_GLOBAL float *mp = as_global<float>(ck.r.m);
    SELSYNC_GLOBAL float *vp = as_global<float>(ck.r.v);
    SELSYNC_GLOBAL uint16_t *cp = as_global<uint16_t>(ck.r.lowp);
    for (uint32_t i = begin + tid; i < end; i += 64) {
        const uint64_t e = ck.off + i;
        float g;
        if (MIXED)
            g = __uint_as_float(((uint32_t)gh[e]) << 16);
        else
            g = gf[e];
        float w = 0.f, m = 0.f, v = 0.f;
        if (UPD) {
            w = wp[e];
            if (OPT::kMomentum && !a.first) {
                m = mp[e];
                if (OPT::kSecondMoment)
                    v = vp[e];
            }
        }
        OPT::template elem<UPD, NORM>(g, w, m, v, a, acc);
        if (UPD) {
            wp[e] = w;
            if (OPT::kMomentum)
                mp[e] = m;
            if (OPT::kSecondMoment)
                vp[e] = v;
            if (MIXED)
                cp[e] = (uint16_t)bf16_bits(w);
        }
    }
}

// Multi-tensor streaming kernel.  Workgroups are single wavefronts (no LDS, no barrier); a
// wavefront takes C table slots that are adjacent in memory, issues the first-tile loads of
// all C chunks before it uses any of them, updates and stores, then (only for chunks larger
// than one tile of 256 elements) walks the remaining tiles.  Per chunk it leaves one fp64
// partial sum of squared scaled gradients in that chunk's slot: fixed place, fixed order, no
// atomics.  The grid is one-shot: workgroup b takes slots (b%8)*per + (b/8)*C + [0, C) of the
// XCD-striped table, so the hardware dispatcher walks the model in order.
// With `pred` set the launch is predicated on a device-side word: it does its work only
// while *pred == pred_want (the gradient-aggregation step runs this kernel on "local" decisions).
template <class OPT, int C, bool MIXED, int MODE, bool NT>
__global__ __launch_bounds__(64) void k_stream(const TensorRec *__restrict__ recs, const ChunkRec *__restrict__ slots,
                                               int nslots, int per, uint32_t chunk_elems,
                                               double *__restrict__ partials, typename OPT::Args a,
                                               const int32_t *__restrict__ pred, int32_t pred_want)
{
    constexpr bool UPD = MODE != kNormOnly;
    constexpr bool NORM = MODE != kUpdateOnly;
    if (pred != nullptr && *pred != pred_want)
        return;
    const uint32_t tid = threadIdx.x;
    const int b = blockIdx.x;
    const int s0 = (b & 7) * per + (b >> 3) * C;
    Chunk ck[C];
    TileRegs t[C];
    double acc[C];
#pragma unroll
    for (int i = 0; i < C; ++i) {
        ck[i] = lookup_chunk(recs, slots, s0 + i, nslots, chunk_elems);
        acc[i] = 0.0;
    }
#pragma unroll
    for (int i = 0; i < C; ++i)
        load_tile<OPT, MIXED, UPD, NT>(ck[i], 0, tid, a.first, t[i]);
#pragma unroll
    for (int i = 0; i < C; ++i)
        finish_tile<OPT, MIXED, UPD, NORM, NT>(ck[i], 0, tid, a, t[i], acc[i]);
#pragma unroll
    for (int i = 0; i < C; ++i) {
        for (uint32_t base = 64; base < ck[i].nvec; base += 64) {
            load_tile<OPT, MIXED, UPD, NT>(ck[i], base, tid, a.first, t[i]);
            finish_tile<OPT, MIXED, UPD, NORM, NT>(ck[i], base, tid, a, t[i], acc[i]);
        }
        scalar_range<OPT, MIXED, UPD, NORM>(ck[i], 0, ck[i].head, tid, a, acc[i]);
        scalar_range<OPT, MIXED, UPD, NORM>(ck[i], ck[i].head + 4 * ck[i].nvec, ck[i].n, tid, a, acc[i]);
    }
    if (NORM) {
#pragma unroll
        for (int i = 0; i < C; ++i) {
            const double s = wave_sum_to_last_lane(acc[i]);
            if (tid == 63 && ck[i].n > 0)
                partials[s0 + i] = s;
        }
    }
}

// ---------------------------------------------------------------- k_reduce

constexpr int kReduceBlock = 256;

// Intermediate level of the deterministic norm reduction: workgroup j sums the per-chunk
// partials of segment j (a fixed range inside one worker's chunks) and writes one value.
// Sum of the partials of chunks b .. e-1 (each in its slot, see chunk_slot) by one workgroup, fixed order: thread-strided accumulation with 8
// independent loads in flight, wavefront shuffle, then the four wave results in wave order.
__device__ __forceinline__ double block_range_sum(const double *__restrict__ partials, int slot_per, int b, int e,
                                                  double *red)
{
    double a8[8] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
    for (int i = b + (int)threadIdx.x; i < e; i += 8 * kReduceBlock) {
        double v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int idx = i + j * kReduceBlock;
            v[j] = idx < e ? partials[chunk_slot(idx, slot_per)] : 0.0;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
            a8[j] += v[j];
    }
    double acc = ((a8[0] + a8[1]) + (a8[2] + a8[3])) + ((a8[4] + a8[5]) + (a8[6] + a8[7]));
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0)
        red[threadIdx.x >> 6] = acc;
    __syncthreads();
    return ((red[0] + red[1]) + red[2]) + red[3];
}

// Per-tensor squared norms from the per-chunk partials of the last tracking pass: workgroup i
// sums the chunk range of one (worker, tensor) pair.
__global__ __launch_bounds__(kReduceBlock) void k_tensor_norms(const double *__restrict__ partials, int slot_per,
                                                               const int32_t *__restrict__ range_begin,
                                                               double *__restrict__ out)
{
    __shared__ double red[kReduceBlock / 64];
    const double s = block_range_sum(partials, slot_per, range_begin[blockIdx.x], range_begin[blockIdx.x + 1], red);
    if (threadIdx.x == 0)
        out[blockIdx.x] = s;
}

__global__ __launch_bounds__(kReduceBlock) void k_reduce(const double *__restrict__ partials, int slot_per,
                                                         const int2 *__restrict__ segs,
                                                         double *__restrict__ seg_sums)
{
    __shared__ double red[kReduceBlock / 64];
    const int2 sg = segs[blockIdx.x];
    const double s = block_range_sum(partials, slot_per, sg.x, sg.y, red);
    if (threadIdx.x == 0)
        seg_sums[blockIdx.x] = s;
}

// ---------------------------------------------------------------- k_track

constexpr int kTrackBlock = 1024;
constexpr int kTrackWaves = kTrackBlock / 64;

// One workgroup handles all K workers, kTrackWaves of them per round.
//   phase 1 (a1, final pass): the waves are split evenly over the workers of the round; each
//     group sums its worker's partials in a fixed order (thread-strided, wave butterfly, then
//     the group's wave results in wave order);
//   phase 2 (a2): wave v owns worker (round*16 + v): one window sample per lane for the
//     weighted sums, lane 0 applies Eq. 2 and the delta rule.
// Afterwards thread 0 ORs the flags (the all-gather of Alg. 1 collapses to this on one
// GPU) and advances the local/sync counters of Eq. 4.
__global__ __launch_bounds__(kTrackBlock) void k_track(TrackerDev td, const double *__restrict__ partials,
                                                       int slot_per, const int32_t *__restrict__ chunk_begin)
{
    __shared__ double s_part[kTrackWaves][kTrackWaves];   // [worker in round][wave]
    __shared__ int32_t s_flag[kTrackWaves];
    __shared__ int32_t s_nonfinite[kTrackWaves];
    __shared__ double s_max[kTrackWaves];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int W = td.window;
    const double thr = *td.delta_thr;
    int32_t my_flag = 0, my_nonfinite = 0;
    double my_max = 0.0;
    // counters are fetched up front so the read-modify-write at the end does not wait on memory
    DecisionHeader hdr{};
    if (threadIdx.x == 0)
        hdr = *td.out;

    for (int k0 = 0; k0 < td.K; k0 += kTrackWaves) {
        const int kn = (td.K - k0) < kTrackWaves ? (td.K - k0) : kTrackWaves;

        // The wave that owns a worker fetches that worker's tracker state and the newest 64 window
        // samples now: these loads do not depend on the norm, so they overlap with phase 1.
        int len = 0, head = 0, len_new = 0, had_prev = 0;
        double pre_v = 0.0, pre_w = 0.0, sp = 0.0;
        if (wave < kn) {
            const int k = k0 + wave;
            len = td.len[k];
            head = td.head[k];
            had_prev = td.has_prev[k];
            sp = td.s_prev[k];
            len_new = len < W ? len + 1 : W;
            if (lane < len_new) {
                pre_w = td.weights[lane];
                if (lane > 0) {
                    int pos = head - lane;
                    if (pos < 0)
                        pos += W;
                    pre_v = td.hist[(size_t)k * W + pos];
                }
            }
        }

        // phase 1: the 16 waves are split evenly over the kn workers of this round, so every worker's
        // partial sums are read at the same time: group r = waves [r*wpw, (r+1)*wpw) strides over worker r's
        // values with 8 independent loads in flight per thread; fixed association order
        const int wpw = kTrackWaves / kn;
        const int r = wave / wpw, wi = wave - r * wpw;
        {
            double acc = 0.0;
            if (r < kn && partials != nullptr) {
                const int b = chunk_begin[k0 + r], e = chunk_begin[k0 + r + 1];
                const int stride = wpw * 64;
                double a8[8] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
                for (int i = b + wi * 64 + lane; i < e; i += 8 * stride) {
                    double v[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const int idx = i + j * stride;
                        v[j] = idx < e ? partials[chunk_slot(idx, slot_per)] : 0.0;
                    }
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        a8[j] += v[j];
                }
                acc = ((a8[0] + a8[1]) + (a8[2] + a8[3])) + ((a8[4] + a8[5]) + (a8[6] + a8[7]));
            }
            acc = wave_sum(acc);
            if (lane == 0 && r < kn)
                s_part[r][wi] = acc;
        }
        __syncthreads();

        if (wave < kn) {
            const int k = k0 + wave;
            double x = 0.0;
            for (int w = 0; w < wpw; ++w)
                x += s_part[wave][w];

            // the window holds the previous `len` samples; the new one has age 0
            double *h = td.hist + (size_t)k * W;
            double num = 0.0, den = 0.0;
            if (lane < len_new) {
                num = pre_w * (lane == 0 ? x : pre_v);
                den = pre_w;
            }
            for (int j = lane + 64; j < len_new; j += 64) {      // windows longer than one wavefront
                const double wgt = td.weights[j];
                int pos = head - j;
                if (pos < 0)
                    pos += W;
                num += wgt * h[pos];
                den += wgt;
            }
            num = wave_sum(num);
            den = wave_sum(den);
            if (lane == 0) {
                const double s = num / den;
                double d;
                if (!had_prev) {
                    d = 0.0;
                } else {
                    if (sp == 0.0 && s == 0.0) {
                        d = 0.0;
                    } else {
                        d = fabs(s - sp) / sp;
                        if (d != d)
                            d = __builtin_inf();
                    }
                }
                const bool finite_x = (x - x) == 0.0;
                if (!finite_x) {
                    d = __builtin_inf();
                    my_nonfinite = 1;
                }
                const int32_t f = (d >= thr) ? 1 : 0;
                my_flag |= f;
                if (d < __builtin_inf() && d > my_max)
                    my_max = d;
                h[head] = x;
                td.head[k] = (head + 1 == W) ? 0 : head + 1;
                td.len[k] = len_new;
                td.s_prev[k] = s;
                td.has_prev[k] = 1;
                td.out_norm_sq[k] = x;
                td.out_delta[k] = d;
                td.out_smoothed[k] = s;
                td.out_flags[k] = f;
            }
        }
        __syncthreads();   // s_part is reused by the next round
    }

    if (lane == 0) {
        s_flag[wave] = my_flag;
        s_nonfinite[wave] = my_nonfinite;
        s_max[wave] = my_max;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t any = 0, nf = 0;
        double mx = hdr.max_delta;
        for (int w = 0; w < kTrackWaves; ++w) {
            any |= s_flag[w];
            nf |= s_nonfinite[w];
            if (s_max[w] > mx)
                mx = s_max[w];
        }
        hdr.sync = any;
        hdr.nonfinite_now = nf;
        hdr.max_delta = mx;
        hdr.nonfinite_steps += nf;
        if (any)
            hdr.steps_sync += 1;
        else
            hdr.steps_local += 1;
        *td.out = hdr;
    }
}

__global__ void k_reset(TrackerDev td)
{
    const int n = td.K * td.window;
    for (int i = threadIdx.x; i < n; i += blockDim.x)
        td.hist[i] = 0.0;
    for (int k = threadIdx.x; k < td.K; k += blockDim.x) {
        td.len[k] = 0;
        td.head[k] = 0;
        td.s_prev[k] = 0.0;
        td.has_prev[k] = 0;
        td.out_norm_sq[k] = 0.0;
        td.out_delta[k] = 0.0;
        td.out_smoothed[k] = 0.0;
        td.out_flags[k] = 0;
    }
    if (threadIdx.x == 0) {
        td.out->steps_local = 0;
        td.out->steps_sync = 0;
        td.out->nonfinite_steps = 0;
        td.out->max_delta = 0.0;
        td.out->sync = 0;
        td.out->nonfinite_now = 0;
    }
}

__global__ void k_set_delta(TrackerDev td, double delta) { *td.delta_thr = delta; }

// Reading order of one worker under DefDP / SelDP (Sec. III-D), written as sample indices.
__global__ __launch_bounds__(256) void k_partition_order(int64_t D, int64_t N, int64_t n, int scheme, int64_t count,
                                                         int64_t *__restrict__ out)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < count; p += stride)
        out[p] = partition_index(D, N, n, scheme, p);
}

// ---------------------------------------------------------------- k_aggregate

// Mean of K fp32 values in fp64, summed k = 0..K-1, divided by K, rounded once to fp32.
// For K a power of two the division is a multiplication by the exact reciprocal.
__device__ __forceinline__ float finish_mean(double s, int K, double invK, int pow2)
{
    const double mean = pow2 ? s * invK : s / (double)K;
    return (float)mean;
}

// Record of the piece that workgroup b works on.  per8 > 0: the table is stored as 8 stripes of per8
// records and piece b sits in stripe b % 8 -- the XCD that workgroup b runs on -- so every table line
// is fetched by one L2 instead of eight while pieces are still dispatched in model order (padding
// records have n = 0).  per8 = 0: plain table.
__device__ __forceinline__ int agg_slot(uint32_t b, int per8)
{
    return per8 > 0 ? (int)(b & 7u) * per8 + (int)(b >> 3) : (int)b;
}

// One workgroup per piece of the aggregation table (one-shot grid).  With mode 0 the launch
// follows the device-side decision: every workgroup reads it and exits at once on "local".
template <int BLOCK, int U, int KC, bool MIXED, bool NT>
__global__ __launch_bounds__(BLOCK) void k_aggregate(const AggChunkRec *__restrict__ chunks, int per8, AggTables tabs,
                                                     int K, double invK, int pow2,
                                                     const int32_t *__restrict__ sync_flag, int mode)
{
    if (mode == 0 && *sync_flag == 0)
        return;
    const uint32_t tid = threadIdx.x;
    {
        const AggChunkRec ch = chunks[agg_slot(blockIdx.x, per8)];
        const uint32_t n = ch.n_flags & kChunkCountMask;
        float *const *wtab = tabs.w + (size_t)ch.t * K;
        uint16_t *const *ctab = MIXED ? tabs.lowp + (size_t)ch.t * K : nullptr;
        SELSYNC_GLOBAL float *gp = as_global<float>(tabs.global[ch.t] + ch.off);
        SELSYNC_GLOBAL uint16_t *gcp = MIXED ? as_global<uint16_t>(tabs.glowp[ch.t] + ch.off) : nullptr;
        uint32_t done = 0;   // elements covered by the 128-bit body [head, head + done)
        uint32_t head = 0;   // elements peeled before it

        if constexpr (KC > 0) {
            // K known at compile time: replica pointers live in registers, all K*U loads
            // of a tile are issued before the first use.
            SELSYNC_GLOBAL float *wp[KC];
            SELSYNC_GLOBAL uint16_t *cp[KC];
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                wp[k] = as_global<float>(wtab[k] + ch.off);
                cp[k] = MIXED ? as_global<uint16_t>(ctab[k] + ch.off) : nullptr;
            }
            if (ch.n_flags & kChunkAligned) {
                head = chunk_head(ch.n_flags, n);
                const uint32_t nvec = (n - head) / 4;
                for (uint32_t base = 0; base < nvec; base += BLOCK * U) {
                    f32x4 v[U][KC];
#pragma unroll
                    for (int k = 0; k < KC; ++k) {
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            const uint32_t i = base + u * BLOCK + tid;
                            v[u][k] = 0.f;
                            if (i < nvec)
                                v[u][k] = ld<NT>((const SELSYNC_GLOBAL f32x4 *)(wp[k] + head) + i);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const uint32_t i = base + u * BLOCK + tid;
                        if (i < nvec) {
                            double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
#pragma unroll
                            for (int k = 0; k < KC; ++k) {
                                s0 += (double)v[u][k].x;
                                s1 += (double)v[u][k].y;
                                s2 += (double)v[u][k].z;
                                s3 += (double)v[u][k].w;
                            }
                            f32x4 r;
                            r.x = finish_mean(s0, KC, invK, pow2);
                            r.y = finish_mean(s1, KC, invK, pow2);
                            r.z = finish_mean(s2, KC, invK, pow2);
                            r.w = finish_mean(s3, KC, invK, pow2);
                            st<NT>((SELSYNC_GLOBAL f32x4 *)(gp + head) + i, r);
                            u32x2 h;
                            if (MIXED) {
                                h.x = bf16_pack(r.x, r.y);
                                h.y = bf16_pack(r.z, r.w);
                                st<NT>((SELSYNC_GLOBAL u32x2 *)(gcp + head) + i, h);
                            }
#pragma unroll
                            for (int k = 0; k < KC; ++k) {
                                st<NT>((SELSYNC_GLOBAL f32x4 *)(wp[k] + head) + i, r);
                                if (MIXED)
                                    st<NT>((SELSYNC_GLOBAL u32x2 *)(cp[k] + head) + i, h);
                            }
                        }
                    }
                }
                done = nvec * 4;
            }
            for (uint32_t j = tid; j < n - done; j += BLOCK) {   // peeled head, then ragged tail
                const uint32_t i = j < head ? j : j + done;
                double s = 0.0;
#pragma unroll
                for (int k = 0; k < KC; ++k)
                    s += (double)wp[k][i];
                const float r = finish_mean(s, KC, invK, pow2);
                gp[i] = r;
                const uint16_t h = MIXED ? (uint16_t)bf16_bits(r) : (uint16_t)0;
                if (MIXED)
                    gcp[i] = h;
#pragma unroll
                for (int k = 0; k < KC; ++k) {
                    wp[k][i] = r;
                    if (MIXED)
                        cp[k][i] = h;
                }
            }
        } else {
            // Any other K: same arithmetic, replica pointers re-read from the table.
            if (ch.n_flags & kChunkAligned) {
                head = chunk_head(ch.n_flags, n);
                const uint32_t nvec = (n - head) / 4;
                for (uint32_t i = tid; i < nvec; i += BLOCK) {
                    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
                    for (int k = 0; k < K; ++k) {
                        const f32x4 v = ld<NT>(as_global<const f32x4>(wtab[k] + ch.off + head) + i);
                        s0 += (double)v.x;
                        s1 += (double)v.y;
                        s2 += (double)v.z;
                        s3 += (double)v.w;
                    }
                    f32x4 r;
                    r.x = finish_mean(s0, K, invK, pow2);
                    r.y = finish_mean(s1, K, invK, pow2);
                    r.z = finish_mean(s2, K, invK, pow2);
                    r.w = finish_mean(s3, K, invK, pow2);
                    st<NT>((SELSYNC_GLOBAL f32x4 *)(gp + head) + i, r);
                    u32x2 h;
                    if (MIXED) {
                        h.x = bf16_pack(r.x, r.y);
                        h.y = bf16_pack(r.z, r.w);
                        st<NT>((SELSYNC_GLOBAL u32x2 *)(gcp + head) + i, h);
                    }
                    for (int k = 0; k < K; ++k) {
                        st<NT>(as_global<f32x4>(wtab[k] + ch.off + head) + i, r);
                        if (MIXED)
                            st<NT>(as_global<u32x2>(ctab[k] + ch.off + head) + i, h);
                    }
                }
                done = nvec * 4;
            }
            for (uint32_t j = tid; j < n - done; j += BLOCK) {   // peeled head, then ragged tail
                const uint32_t i = j < head ? j : j + done;
                double s = 0.0;
                for (int k = 0; k < K; ++k)
                    s += (double)as_global<const float>(wtab[k])[ch.off + i];
                const float r = finish_mean(s, K, invK, pow2);
                gp[i] = r;
                const uint16_t h = MIXED ? (uint16_t)bf16_bits(r) : (uint16_t)0;
                if (MIXED)
                    gcp[i] = h;
                for (int k = 0; k < K; ++k) {
                    as_global<float>(wtab[k])[ch.off + i] = r;
                    if (MIXED)
                        as_global<uint16_t>(ctab[k])[ch.off + i] = h;
                }
            }
        }
    }
}

// ---------------------------------------------------------------- k_update_ga

// One gradient element: fp32, or bf16 widened exactly.
template <bool MIXED>
__device__ __forceinline__ float load_grad(const void *g, uint64_t e)
{
    if (MIXED)
        return __uint_as_float(((uint32_t)as_global<const uint16_t>(g)[e]) << 16);
    return as_global<const float>(g)[e];
}

// Mean of K scaled gradients, fp64 sum in worker order, one rounding to fp32.
template <int KC>
__device__ __forceinline__ f32x4 mean_grad4(const f32x4 *g, int K, float gs, double invK, int pow2)
{
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    const int n = KC > 0 ? KC : K;
    for (int k = 0; k < n; ++k) {
        const float a0 = gs * g[k].x, a1 = gs * g[k].y, a2 = gs * g[k].z, a3 = gs * g[k].w;
        s0 += (double)a0;
        s1 += (double)a1;
        s2 += (double)a2;
        s3 += (double)a3;
    }
    f32x4 r;
    r.x = finish_mean(s0, n, invK, pow2);
    r.y = finish_mean(s1, n, invK, pow2);
    r.z = finish_mean(s2, n, invK, pow2);
    r.w = finish_mean(s3, n, invK, pow2);
    return r;
}

// The synchronising update of gradient aggregation (Sec. III-C): one workgroup walks one
// piece of one tensor across the K workers and applies the mean gradient to every worker's
// own state with the optimiser policy OPT (momentum SGD, momentum-free SGD, Adam: the
// moment buffers stay per worker).  Launched on every step of that variant.  `mode` says what
// the launch does with the device-side decision:
//   kGaAlways         aggregate whatever the decision is;
//   kGaSyncOnly       aggregate on "sync", exit at once on "local" (the plain local update of such
//                     a step is then the streaming kernel's job, in its own predicated launch);
//   kGaSyncOrLocal    aggregate on "sync"; on "local" every worker applies its OWN gradient, here
//                     (one launch serves both decisions: for steps that are expected to synchronise).
// K compile-time (KC > 0) keeps all loads of a vector in flight.
template <class OPT, int BLOCK, int KC, bool MIXED, bool NT>
__global__ __launch_bounds__(BLOCK) void k_update_ga(const AggChunkRec *__restrict__ chunks, int per8, AggTables tabs,
                                                     int K, double invK, int pow2,
                                                     const int32_t *__restrict__ sync_flag, int mode,
                                                     typename OPT::Args a)
{
    constexpr int KM = KC > 0 ? KC : 1;
    const bool sync = mode == kGaAlways || *sync_flag != 0;
    if (!sync && mode == kGaSyncOnly)
        return;
    typename OPT::Args a1 = a;   // applied to the mean gradient, which is already scaled
    a1.gs = 1.f;
    const uint32_t tid = threadIdx.x;
    double unused = 0.0;
    {
        const AggChunkRec ch = chunks[agg_slot(blockIdx.x, per8)];
        const uint32_t n = ch.n_flags & kChunkCountMask;
        const size_t row = (size_t)ch.t * K;
        uint32_t done = 0;   // elements covered by the 128-bit body [head, head + done)
        uint32_t head = 0;
        if constexpr (KC > 0) {
            if ((ch.n_flags & kChunkAligned) && (ch.n_flags & kChunkAlignedGrads)) {
                head = chunk_head(ch.n_flags, n);
                const uint64_t off = ch.off + head;
                SELSYNC_GLOBAL f32x4 *wp[KM];
                SELSYNC_GLOBAL f32x4 *mp[KM];
                SELSYNC_GLOBAL f32x4 *vp[KM];
                const SELSYNC_GLOBAL f32x4 *gp[KM];
                const SELSYNC_GLOBAL u32x2 *gbp[KM];
                SELSYNC_GLOBAL u32x2 *cp[KM];
#pragma unroll
                for (int k = 0; k < KC; ++k) {
                    wp[k] = as_global<f32x4>(tabs.w[row + k] + off);
                    mp[k] = OPT::kMomentum ? as_global<f32x4>(tabs.m[row + k] + off) : nullptr;
                    vp[k] = OPT::kSecondMoment ? as_global<f32x4>(tabs.v[row + k] + off) : nullptr;
                    gp[k] = MIXED ? nullptr : as_global<const f32x4>(static_cast<const float *>(tabs.g[row + k]) + off);
                    gbp[k] = MIXED ? as_global<const u32x2>(static_cast<const uint16_t *>(tabs.g[row + k]) + off)
                                   : nullptr;
                    cp[k] = MIXED ? as_global<u32x2>(tabs.lowp[row + k] + off) : nullptr;
                }
                const uint32_t nvec = (n - head) / 4;
                for (uint32_t i = tid; i < nvec; i += BLOCK) {
                    f32x4 gv[KM], wv[KM], mv[KM], vv[KM];
#pragma unroll
                    for (int k = 0; k < KC; ++k) {
                        if (MIXED)
                            gv[k] = widen4(ld<NT>(gbp[k] + i));
                        else
                            gv[k] = ld<NT>(gp[k] + i);
                        wv[k] = ld<NT>(wp[k] + i);
                        mv[k] = 0.f;
                        vv[k] = 0.f;
                        if (OPT::kMomentum && !a.first) {
                            mv[k] = ld<NT>(mp[k] + i);
                            if (OPT::kSecondMoment)
                                vv[k] = ld<NT>(vp[k] + i);
                        }
                    }
                    f32x4 gbar = 0.f;
                    if (sync)
                        gbar = mean_grad4<KC>(gv, KC, a.gs, invK, pow2);
#pragma unroll
                    for (int k = 0; k < KC; ++k) {
                        if (sync)
                            elem4<OPT, true, false>(gbar, wv[k], mv[k], vv[k], a1, unused);
                        else
                            elem4<OPT, true, false>(gv[k], wv[k], mv[k], vv[k], a, unused);
                        st<NT>(wp[k] + i, wv[k]);
                        if (OPT::kMomentum)
                            st<NT>(mp[k] + i, mv[k]);
                        if (OPT::kSecondMoment)
                            st<NT>(vp[k] + i, vv[k]);
                        if (MIXED) {
                            u32x2 cv;
                            cv.x = bf16_pack(wv[k].x, wv[k].y);
                            cv.y = bf16_pack(wv[k].z, wv[k].w);
                            st<NT>(cp[k] + i, cv);
                        }
                    }
                }
                done = nvec * 4;
            }
        }
        // element-at-a-time: unaligned tensors, ragged tails, and any K without a compiled shape
        for (uint32_t j = tid; j < n - done; j += BLOCK) {
            const uint32_t i = j < head ? j : j + done;
            const uint64_t e = ch.off + i;
            double s = 0.0;
            if (sync) {
                for (int k = 0; k < K; ++k) {
                    const float gh = a.gs * load_grad<MIXED>(tabs.g[row + k], e);
                    s += (double)gh;
                }
            }
            const float gbar = finish_mean(s, K, invK, pow2);
            for (int k = 0; k < K; ++k) {
                SELSYNC_GLOBAL float *wq = as_global<float>(tabs.w[row + k]);
                float w = wq[e];
                float m = 0.f, v = 0.f;
                if (OPT::kMomentum && !a.first) {
                    m = as_global<const float>(tabs.m[row + k])[e];
                    if (OPT::kSecondMoment)
                        v = as_global<const float>(tabs.v[row + k])[e];
                }
                if (sync)
                    OPT::template elem<true, false>(gbar, w, m, v, a1, unused);
                else
                    OPT::template elem<true, false>(load_grad<MIXED>(tabs.g[row + k], e), w, m, v, a, unused);
                wq[e] = w;
                if (OPT::kMomentum)
                    as_global<float>(tabs.m[row + k])[e] = m;
                if (OPT::kSecondMoment)
                    as_global<float>(tabs.v[row + k])[e] = v;
                if (MIXED)
                    as_global<uint16_t>(tabs.lowp[row + k])[e] = (uint16_t)bf16_bits(w);
            }
        }
    }
}

// ---------------------------------------------------------------- k_sync_step

// A whole fully synchronous iteration in ONE pass (a threshold of 0 turns SelSync into BSP,
// Sec. III-B): for one 256-element piece of one tensor across all K workers, a single
// wavefront reads every worker's g, w, m once, accumulates each worker's squared scaled
// gradient (Alg. 1 line 8), applies each worker's local update (line 9), forms the mean of
// the updated parameters in fp64 in worker order (lines 14-15) and writes it to every
// replica and the global model, and each worker's new momentum to its buffer:
// 20*K + 4 bytes per parameter instead of the 28*K + 4 of update pass + aggregation pass
// (with Adam as the update: 28*K + 4 instead of 36*K + 4; the moment buffers stay per worker).
// Arithmetic, rounding sequence and sum orders are those of k_stream and k_aggregate, so
// the tensors are bit-identical to the two-pass sequence.  Per (worker, piece) it leaves one
// fp64 partial, formed in the order k_stream uses for a chunk (vector body, peeled head, ragged
// tail; DPP wavefront sum).  The partials are striped by XCD like the table: with worker k's
// pieces numbered c = k * 8 * per8 + piece, partial c sits at (c % 8) * (K * per8) + c / 8, so the
// eight-byte results of one XCD's wavefronts share cache lines with each other only.
template <class OPT, int KC, bool MIXED, bool NT>
__global__ __launch_bounds__(64) void k_sync_step(const AggChunkRec *__restrict__ chunks, int per8, AggTables tabs,
                                                  int K, double invK, int pow2, typename OPT::Args a,
                                                  double *__restrict__ partials)
{
    constexpr int KM = KC > 0 ? KC : 1;
    const uint32_t tid = threadIdx.x;
    const AggChunkRec ch = chunks[agg_slot(blockIdx.x, per8)];
    // slot of worker 0's partial for this piece; worker k's lies k * per8 further on
    const size_t pslot = (size_t)(blockIdx.x & 7u) * ((size_t)K * per8) + (blockIdx.x >> 3);
    const uint32_t n = ch.n_flags & kChunkCountMask;
    const size_t row = (size_t)ch.t * K;
    SELSYNC_GLOBAL float *gl = as_global<float>(tabs.global[ch.t]);
    SELSYNC_GLOBAL uint16_t *glc = MIXED ? as_global<uint16_t>(tabs.glowp[ch.t]) : nullptr;
    const bool vec = (ch.n_flags & kChunkAligned) && (ch.n_flags & kChunkAlignedGrads);
    const uint32_t head = vec ? chunk_head(ch.n_flags, n) : 0u;
    const uint32_t nvec = vec ? (n - head) / 4 : 0u;          // <= 64: a piece holds at most 256 elements
    const uint64_t e0 = ch.off + head;
    const bool lane_vec = tid < nvec;

    if constexpr (KC > 0) {
        double acc[KM];
        f32x4 gv[KM], wv[KM], mv[KM], vv[KM];
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            acc[k] = 0.0;
            gv[k] = 0.f;
            wv[k] = 0.f;
            mv[k] = 0.f;
            vv[k] = 0.f;
            if (lane_vec) {
                if (MIXED)
                    gv[k] = widen4(ld<NT>(as_global<const u32x2>(static_cast<const uint16_t *>(tabs.g[row + k]) + e0) + tid));
                else
                    gv[k] = ld<NT>(as_global<const f32x4>(static_cast<const float *>(tabs.g[row + k]) + e0) + tid);
                wv[k] = ld<NT>(as_global<const f32x4>(tabs.w[row + k] + e0) + tid);
                if (OPT::kMomentum && !a.first) {
                    mv[k] = ld<NT>(as_global<const f32x4>(tabs.m[row + k] + e0) + tid);
                    if (OPT::kSecondMoment)
                        vv[k] = ld<NT>(as_global<const f32x4>(tabs.v[row + k] + e0) + tid);
                }
            }
        }
        if (lane_vec) {
            double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                elem4<OPT, true, true>(gv[k], wv[k], mv[k], vv[k], a, acc[k]);
                s0 += (double)wv[k].x;
                s1 += (double)wv[k].y;
                s2 += (double)wv[k].z;
                s3 += (double)wv[k].w;
                if (OPT::kMomentum)
                    st<NT>(as_global<f32x4>(tabs.m[row + k] + e0) + tid, mv[k]);
                if (OPT::kSecondMoment)
                    st<NT>(as_global<f32x4>(tabs.v[row + k] + e0) + tid, vv[k]);
            }
            f32x4 r;
            r.x = finish_mean(s0, KC, invK, pow2);
            r.y = finish_mean(s1, KC, invK, pow2);
            r.z = finish_mean(s2, KC, invK, pow2);
            r.w = finish_mean(s3, KC, invK, pow2);
            u32x2 h;
            if (MIXED) {
                h.x = bf16_pack(r.x, r.y);
                h.y = bf16_pack(r.z, r.w);
            }
            st<NT>((SELSYNC_GLOBAL f32x4 *)(gl + e0) + tid, r);
            if (MIXED)
                st<NT>((SELSYNC_GLOBAL u32x2 *)(glc + e0) + tid, h);
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                st<NT>(as_global<f32x4>(tabs.w[row + k] + e0) + tid, r);
                if (MIXED)
                    st<NT>(as_global<u32x2>(tabs.lowp[row + k] + e0) + tid, h);
            }
        }
        // peeled head, then ragged tail (all of the piece when its streams are not vector-aligned together);
        // lane i takes element begin + i of either range, as in k_stream, so the partial sums group alike
        auto scalar_elem = [&](uint64_t e) {
            double s = 0.0;
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                float g;
                if (MIXED)
                    g = __uint_as_float(((uint32_t)as_global<const uint16_t>(tabs.g[row + k])[e]) << 16);
                else
                    g = as_global<const float>(tabs.g[row + k])[e];
                float w = as_global<const float>(tabs.w[row + k])[e];
                float m = 0.f, v = 0.f;
                if (OPT::kMomentum && !a.first) {
                    m = as_global<const float>(tabs.m[row + k])[e];
                    if (OPT::kSecondMoment)
                        v = as_global<const float>(tabs.v[row + k])[e];
                }
                OPT::template elem<true, true>(g, w, m, v, a, acc[k]);
                s += (double)w;
                if (OPT::kMomentum)
                    as_global<float>(tabs.m[row + k])[e] = m;
                if (OPT::kSecondMoment)
                    as_global<float>(tabs.v[row + k])[e] = v;
            }
            const float r = finish_mean(s, KC, invK, pow2);
            const uint16_t h = MIXED ? (uint16_t)bf16_bits(r) : (uint16_t)0;
            gl[e] = r;
            if (MIXED)
                glc[e] = h;
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                as_global<float>(tabs.w[row + k])[e] = r;
                if (MIXED)
                    as_global<uint16_t>(tabs.lowp[row + k])[e] = h;
            }
        };
        const uint32_t done = nvec * 4;
        for (uint32_t i = tid; i < head; i += 64)
            scalar_elem(ch.off + i);
        for (uint32_t i = head + done + tid; i < n; i += 64)
            scalar_elem(ch.off + i);
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            const double x = wave_sum_to_last_lane(acc[k]);
            if (tid == 63 && n > 0)
                partials[pslot + (size_t)k * per8] = x;
        }
    } else {
        // Any other K: the same arithmetic with one worker in registers at a time.  Lane `tid` owns vector
        // `tid` of the body and elements tid, tid + 64, ... of head and tail; every worker's contribution to
        // a lane's fp64 sums arrives in worker order.
        const uint32_t done = nvec * 4;
        uint32_t nsc = 0;                       // scalar elements of this lane (at most 4: a piece has <= 256)
        uint64_t se[4];
        if (tid < head)
            se[nsc++] = ch.off + tid;
        for (uint32_t i = head + done + tid; i < n && nsc < 4; i += 64)
            se[nsc++] = ch.off + i;
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
        double ss[4] = {0.0, 0.0, 0.0, 0.0};
        for (int k = 0; k < K; ++k) {
            double acc = 0.0;
            if (lane_vec) {
                f32x4 gv, wv, mv = 0.f, vv = 0.f;
                if (MIXED)
                    gv = widen4(ld<NT>(as_global<const u32x2>(static_cast<const uint16_t *>(tabs.g[row + k]) + e0) + tid));
                else
                    gv = ld<NT>(as_global<const f32x4>(static_cast<const float *>(tabs.g[row + k]) + e0) + tid);
                wv = ld<NT>(as_global<const f32x4>(tabs.w[row + k] + e0) + tid);
                if (OPT::kMomentum && !a.first) {
                    mv = ld<NT>(as_global<const f32x4>(tabs.m[row + k] + e0) + tid);
                    if (OPT::kSecondMoment)
                        vv = ld<NT>(as_global<const f32x4>(tabs.v[row + k] + e0) + tid);
                }
                elem4<OPT, true, true>(gv, wv, mv, vv, a, acc);
                s0 += (double)wv.x;
                s1 += (double)wv.y;
                s2 += (double)wv.z;
                s3 += (double)wv.w;
                if (OPT::kMomentum)
                    st<NT>(as_global<f32x4>(tabs.m[row + k] + e0) + tid, mv);
                if (OPT::kSecondMoment)
                    st<NT>(as_global<f32x4>(tabs.v[row + k] + e0) + tid, vv);
            }
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q) {
                if (q < nsc) {
                    const uint64_t e = se[q];
                    float g;
                    if (MIXED)
                        g = __uint_as_float(((uint32_t)as_global<const uint16_t>(tabs.g[row + k])[e]) << 16);
                    else
                        g = as_global<const float>(tabs.g[row + k])[e];
                    float w = as_global<const float>(tabs.w[row + k])[e];
                    float m = 0.f, v = 0.f;
                    if (OPT::kMomentum && !a.first) {
                        m = as_global<const float>(tabs.m[row + k])[e];
                        if (OPT::kSecondMoment)
                            v = as_global<const float>(tabs.v[row + k])[e];
                    }
                    OPT::template elem<true, true>(g, w, m, v, a, acc);
                    ss[q] += (double)w;
                    if (OPT::kMomentum)
                        as_global<float>(tabs.m[row + k])[e] = m;
                    if (OPT::kSecondMoment)
                        as_global<float>(tabs.v[row + k])[e] = v;
                }
            }
            const double x = wave_sum_to_last_lane(acc);
            if (tid == 63 && n > 0)
                partials[pslot + (size_t)k * per8] = x;
        }
        f32x4 r = 0.f;
        u32x2 h = 0u;
        if (lane_vec) {
            r.x = finish_mean(s0, K, invK, pow2);
            r.y = finish_mean(s1, K, invK, pow2);
            r.z = finish_mean(s2, K, invK, pow2);
            r.w = finish_mean(s3, K, invK, pow2);
            if (MIXED) {
                h.x = bf16_pack(r.x, r.y);
                h.y = bf16_pack(r.z, r.w);
            }
            st<NT>((SELSYNC_GLOBAL f32x4 *)(gl + e0) + tid, r);
            if (MIXED)
                st<NT>((SELSYNC_GLOBAL u32x2 *)(glc + e0) + tid, h);
        }
        float rs[4];
        uint16_t hs[4];
#pragma unroll
        for (uint32_t q = 0; q < 4; ++q) {
            rs[q] = 0.f;
            hs[q] = 0;
            if (q < nsc) {
                rs[q] = finish_mean(ss[q], K, invK, pow2);
                hs[q] = MIXED ? (uint16_t)bf16_bits(rs[q]) : (uint16_t)0;
                gl[se[q]] = rs[q];
                if (MIXED)
                    glc[se[q]] = hs[q];
            }
        }
        for (int k = 0; k < K; ++k) {
            if (lane_vec) {
                st<NT>(as_global<f32x4>(tabs.w[row + k] + e0) + tid, r);
                if (MIXED)
                    st<NT>(as_global<u32x2>(tabs.lowp[row + k] + e0) + tid, h);
            }
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q) {
                if (q < nsc) {
                    as_global<float>(tabs.w[row + k])[se[q]] = rs[q];
                    if (MIXED)
                        as_global<uint16_t>(tabs.lowp[row + k])[se[q]] = hs[q];
                }
            }
        }
    }
}

// ---------------------------------------------------------------- dispatch helpers

// Chunks per wavefront of the streaming kernel (measured on the 133M-parameter fp32 workload):
// updates do best with the least work per wavefront, one chunk; the read-only norm pass wants
// more bytes in flight per wavefront, four chunks.
constexpr int kUpdateChunksPerWave = 1;
constexpr int kNormChunksPerWave = 4;
static_assert(kStripeGranule % kNormChunksPerWave == 0 && kStripeGranule % kUpdateChunksPerWave == 0,
              "a wavefront's slots must not cross a stripe");

template <class OPT, int C, bool MIXED, int MODE, bool NT>
hipError_t launch_stream_c(const StreamTable &tab, const typename OPT::Args &args, const int32_t *pred, int pred_want,
                           hipStream_t s)
{
    const int nwg = 8 * (tab.per / C);
    hipLaunchKernelGGL((k_stream<OPT, C, MIXED, MODE, NT>), dim3(nwg), dim3(64), 0, s, tab.recs, tab.slots, tab.nslots,
                       tab.per, tab.chunk_elems, tab.partials, args, pred, pred_want);
    return hipGetLastError();
}

template <class OPT, bool MIXED, bool NT>
hipError_t launch_stream_m(StreamMode mode, const StreamTable &tab, const typename OPT::Args &args,
                           const int32_t *pred, int pred_want, hipStream_t s)
{
    switch (mode) {
    case kNormOnly:
        return launch_stream_c<OPT, kNormChunksPerWave, MIXED, kNormOnly, NT>(tab, args, pred, pred_want, s);
    case kUpdateOnly:
        return launch_stream_c<OPT, kUpdateChunksPerWave, MIXED, kUpdateOnly, NT>(tab, args, pred, pred_want, s);
    default:
        return launch_stream_c<OPT, kUpdateChunksPerWave, MIXED, kUpdateAndNorm, NT>(tab, args, pred, pred_want, s);
    }
}

template <class OPT>
hipError_t launch_stream_o(StreamMode mode, bool mixed, const StreamTable &tab, const typename OPT::Args &args,
                           bool nontemporal, const int32_t *pred, int pred_want, hipStream_t s)
{
    if (tab.nchunks <= 0)
        return hipSuccess;
    if (mixed)
        return nontemporal ? launch_stream_m<OPT, true, true>(mode, tab, args, pred, pred_want, s)
                           : launch_stream_m<OPT, true, false>(mode, tab, args, pred, pred_want, s);
    return nontemporal ? launch_stream_m<OPT, false, true>(mode, tab, args, pred, pred_want, s)
                       : launch_stream_m<OPT, false, false>(mode, tab, args, pred, pred_want, s);
}

// The two shapes of the K-way kernels: kAggCoarse for launches that follow the device-side decision
// (few, large workgroups: cheap to dispatch when they only read the decision and exit), kAggFine for
// launches over 256-element pieces (one wavefront, one 128-bit access per lane and stream).
template <int KC, bool MIXED, bool NT>
hipError_t launch_agg_t(const AggTable &t, const AggTables &tabs, int K, const int32_t *flag, int mode, hipStream_t s)
{
    const int pow2 = (K & (K - 1)) == 0;
    if (t.shape == kAggFine)
        hipLaunchKernelGGL((k_aggregate<64, 1, KC, MIXED, NT>), dim3(t.nslots), dim3(64), 0, s, t.recs, t.per8, tabs, K,
                           1.0 / (double)K, pow2, flag, mode);
    else
        hipLaunchKernelGGL((k_aggregate<256, 4, KC, MIXED, NT>), dim3(t.nslots), dim3(256), 0, s, t.recs, t.per8, tabs,
                           K, 1.0 / (double)K, pow2, flag, mode);
    return hipGetLastError();
}

template <class OPT, int KC, bool MIXED, bool NT>
hipError_t launch_ga_t(const AggTable &t, const AggTables &tabs, int K, const int32_t *flag, int mode,
                       const typename OPT::Args &args, hipStream_t s)
{
    const int pow2 = (K & (K - 1)) == 0;
    if (t.shape == kAggFine)
        hipLaunchKernelGGL((k_update_ga<OPT, 64, KC, MIXED, NT>), dim3(t.nslots), dim3(64), 0, s, t.recs, t.per8, tabs,
                           K, 1.0 / (double)K, pow2, flag, mode, args);
    else
        hipLaunchKernelGGL((k_update_ga<OPT, 256, KC, MIXED, NT>), dim3(t.nslots), dim3(256), 0, s, t.recs, t.per8, tabs,
                           K, 1.0 / (double)K, pow2, flag, mode, args);
    return hipGetLastError();
}

// Compile-time worker counts of the K-way kernels (replica pointers in registers); any other K
// takes the run-time-K path (KC = 0).
#define SELSYNC_SWITCH_K(K, CALL)      \
    switch (K) {                       \
    case 1: return CALL(1);            \
    case 2: return CALL(2);            \
    case 4: return CALL(4);            \
    case 8: return CALL(8);            \
    default: return CALL(0);           \
    }

template <bool MIXED, bool NT>
hipError_t launch_agg_k(const AggTable &t, const AggTables &tabs, int K, const int32_t *flag, int mode, hipStream_t s)
{
#define SELSYNC_AGG_CALL(KC) launch_agg_t<KC, MIXED, NT>(t, tabs, K, flag, mode, s)
    SELSYNC_SWITCH_K(K, SELSYNC_AGG_CALL)
#undef SELSYNC_AGG_CALL
}

template <class OPT, bool MIXED, bool NT>
hipError_t launch_ga_k(const AggTable &t, const AggTables &tabs, int K, const int32_t *flag, int mode,
                       const typename OPT::Args &args, hipStream_t s)
{
#define SELSYNC_GA_CALL(KC) launch_ga_t<OPT, KC, MIXED, NT>(t, tabs, K, flag, mode, args, s)
    SELSYNC_SWITCH_K(K, SELSYNC_GA_CALL)
#undef SELSYNC_GA_CALL
}

template <class OPT>
hipError_t launch_ga_o(bool mixed, const AggTable &t, const AggTables &tabs, int K, const int32_t *flag, int mode,
                       const typename OPT::Args &args, bool nontemporal, hipStream_t s)
{
    if (t.nslots <= 0)
        return hipSuccess;
    if (mixed)
        return nontemporal ? launch_ga_k<OPT, true, true>(t, tabs, K, flag, mode, args, s)
                           : launch_ga_k<OPT, true, false>(t, tabs, K, flag, mode, args, s);
    return nontemporal ? launch_ga_k<OPT, false, true>(t, tabs, K, flag, mode, args, s)
                       : launch_ga_k<OPT, false, false>(t, tabs, K, flag, mode, args, s);
}

template <class OPT, int KC, bool MIXED, bool NT>
hipError_t launch_sync_t(const AggTable &t, const AggTables &tabs, int K, const typename OPT::Args &sgd, double *partials,
                         hipStream_t s)
{
    const int pow2 = (K & (K - 1)) == 0;
    hipLaunchKernelGGL((k_sync_step<OPT, KC, MIXED, NT>), dim3(t.nslots), dim3(64), 0, s, t.recs, t.per8, tabs, K,
                       1.0 / (double)K, pow2, sgd, partials);
    return hipGetLastError();
}

template <class OPT, bool MIXED, bool NT>
hipError_t launch_sync_k(const AggTable &t, const AggTables &tabs, int K, const typename OPT::Args &sgd, double *partials,
                         hipStream_t s)
{
#define SELSYNC_SYNC_CALL(KC) launch_sync_t<OPT, KC, MIXED, NT>(t, tabs, K, sgd, partials, s)
    SELSYNC_SWITCH_K(K, SELSYNC_SYNC_CALL)
#undef SELSYNC_SYNC_CALL
}

template <class OPT>
hipError_t launch_sync_o(bool mixed, const AggTable &t, const AggTables &tabs, int K, const typename OPT::Args &sgd,
                         double *partials, bool nontemporal, hipStream_t s)
{
    if (t.nslots <= 0)
        return hipSuccess;
    if (mixed)
        return nontemporal ? launch_sync_k<OPT, true, true>(t, tabs, K, sgd, partials, s)
                           : launch_sync_k<OPT, true, false>(t, tabs, K, sgd, partials, s);
    return nontemporal ? launch_sync_k<OPT, false, true>(t, tabs, K, sgd, partials, s)
                       : launch_sync_k<OPT, false, false>(t, tabs, K, sgd, partials, s);
}

}  // namespace

// ---------------------------------------------------------------- launchers

hipError_t launch_stream(StreamMode mode, bool mixed, const StreamTable &tab, const SgdArgs &sgd, bool nontemporal,
                         hipStream_t s, const int32_t *pred, int pred_want)
{
    if (!tab.has_momentum)
        return launch_stream_o<PlainSgdOpt>(mode, mixed, tab, sgd, nontemporal, pred, pred_want, s);
    return launch_stream_o<SgdOpt>(mode, mixed, tab, sgd, nontemporal, pred, pred_want, s);
}

hipError_t launch_stream_adam(bool with_norm, bool mixed, const StreamTable &tab, const AdamArgs &a, bool nontemporal,
                              hipStream_t s, const int32_t *pred, int pred_want)
{
    return launch_stream_o<AdamOpt>(with_norm ? kUpdateAndNorm : kUpdateOnly, mixed, tab, a, nontemporal, pred,
                                    pred_want, s);
}

hipError_t launch_reduce(const double *partials, int slot_per, const int2 *segs, int nsegs, double *seg_sums,
                         hipStream_t s)
{
    if (nsegs <= 0)
        return hipSuccess;
    hipLaunchKernelGGL(k_reduce, dim3(nsegs), dim3(kReduceBlock), 0, s, partials, slot_per, segs, seg_sums);
    return hipGetLastError();
}

hipError_t launch_tensor_norms(const double *partials, int slot_per, const int32_t *range_begin, int nranges,
                               double *out, hipStream_t s)
{
    if (nranges <= 0)
        return hipSuccess;
    hipLaunchKernelGGL(k_tensor_norms, dim3(nranges), dim3(kReduceBlock), 0, s, partials, slot_per, range_begin, out);
    return hipGetLastError();
}

hipError_t launch_track(const TrackerDev &td, const double *values, int slot_per, const int32_t *begin, hipStream_t s)
{
    hipLaunchKernelGGL(k_track, dim3(1), dim3(kTrackBlock), 0, s, td, values, slot_per, begin);
    return hipGetLastError();
}

hipError_t launch_aggregate(bool mixed, const AggTable &t, const AggTables &tabs, int K, const int32_t *sync_flag,
                            int mode, bool nontemporal, hipStream_t s)
{
    if (t.nslots <= 0)
        return hipSuccess;
    if (mixed)
        return nontemporal ? launch_agg_k<true, true>(t, tabs, K, sync_flag, mode, s)
                           : launch_agg_k<true, false>(t, tabs, K, sync_flag, mode, s);
    return nontemporal ? launch_agg_k<false, true>(t, tabs, K, sync_flag, mode, s)
                       : launch_agg_k<false, false>(t, tabs, K, sync_flag, mode, s);
}

hipError_t launch_update_ga(bool mixed, bool has_momentum, const AggTable &t, const AggTables &tabs, int K,
                            const int32_t *sync_flag, int mode, const SgdArgs &sgd, bool nontemporal, hipStream_t s)
{
    if (!has_momentum)
        return launch_ga_o<PlainSgdOpt>(mixed, t, tabs, K, sync_flag, mode, sgd, nontemporal, s);
    return launch_ga_o<SgdOpt>(mixed, t, tabs, K, sync_flag, mode, sgd, nontemporal, s);
}

hipError_t launch_update_ga_adam(bool mixed, const AggTable &t, const AggTables &tabs, int K, const int32_t *sync_flag,
                                 int mode, const AdamArgs &a, bool nontemporal, hipStream_t s)
{
    return launch_ga_o<AdamOpt>(mixed, t, tabs, K, sync_flag, mode, a, nontemporal, s);
}

hipError_t launch_sync_step(bool mixed, bool has_momentum, const AggTable &t, const AggTables &tabs, int K,
                            const SgdArgs &sgd, double *partials, bool nontemporal, hipStream_t s)
{
    if (t.nslots <= 0)
        return hipSuccess;
    if (!has_momentum)
        return launch_sync_o<PlainSgdOpt>(mixed, t, tabs, K, sgd, partials, nontemporal, s);
    return launch_sync_o<SgdOpt>(mixed, t, tabs, K, sgd, partials, nontemporal, s);
}

hipError_t launch_sync_step_adam(bool mixed, const AggTable &t, const AggTables &tabs, int K, const AdamArgs &a,
                                 double *partials, bool nontemporal, hipStream_t s)
{
    return launch_sync_o<AdamOpt>(mixed, t, tabs, K, a, partials, nontemporal, s);
}

hipError_t launch_partition_order(int64_t D, int64_t N, int64_t n, int scheme, int64_t count, int64_t *out,
                                  hipStream_t s)
{
    if (count <= 0)
        return hipSuccess;
    const int64_t blocks = (count + 255) / 256;
    const int grid = (int)(blocks < 65536 ? blocks : 65536);
    hipLaunchKernelGGL(k_partition_order, dim3(grid), dim3(256), 0, s, D, N, n, scheme, count, out);
    return hipGetLastError();
}

hipError_t launch_reset(const TrackerDev &td, hipStream_t s)
{
    hipLaunchKernelGGL(k_reset, dim3(1), dim3(256), 0, s, td);
    return hipGetLastError();
}

hipError_t launch_set_delta(const TrackerDev &td, double delta, hipStream_t s)
{
    hipLaunchKernelGGL(k_set_delta, dim3(1), dim3(1), 0, s, td, delta);
    return hipGetLastError();
}

}  // namespace selsync
