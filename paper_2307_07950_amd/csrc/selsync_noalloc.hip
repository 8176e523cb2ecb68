// Entry point for callers that cannot allocate device memory (code under HIP graph capture,
// tight serving loops, harnesses that forbid hipMalloc): the squared gradient norms of K
// workers -- the a1 part of selsync_track_grad_change (Alg. 1 line 8) -- with no context,
// no plan and no allocation.  The per-piece partial sums, which a plan keeps in memory it
// allocates, live here in a file-scope device array (`scratch`), one copy per GPU.
//
// Tensor descriptors travel to the device inside the kernel arguments, kBatch at a time;
// every piece of kPiece elements has a fixed slot in `scratch` and every sum a fixed
// order, so the result is the same on every run.  A final launch adds each worker's range
// of slots and writes x_k to the caller's device array.
#include "../../include/selsync.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kPiece = 4096;            // elements per piece: 256 threads x 4 vectors of 4 elements
constexpr int kBlock = 256;
constexpr int kBatch = 64;              // tensor descriptors per launch (they ride in the kernel arguments)
constexpr int kMaxPieces = 1 << 20;     // slots in `scratch`: 8 MiB, 2^32 elements over all workers per call
constexpr int kMaxWorkersNoAlloc = 64;  // worker ranges ride in the kernel arguments of the final launch
constexpr int kMaxDevices = 64;

// One fp64 partial sum per piece.  Shared by every call on a GPU: calls that overlap on one GPU race.
// Nothing in it has to start at zero: a call writes every slot it later reads.
static __device__ __align__(256) double scratch[kMaxPieces];

struct Batch {
    const void *ptr[kBatch];
    int64_t numel[kBatch];
    int32_t first_piece[kBatch + 1];   // piece index (inside this launch) at which tensor d starts
    int32_t count;                     // tensors in this launch
    int32_t slot0;                     // slot in `scratch` of this launch's piece 0
};

struct Ranges {
    int32_t begin[kMaxWorkersNoAlloc + 1];   // worker k's slots are [begin[k], begin[k+1])
};

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        v += __shfl_down(v, o, 64);
    return v;
}

// Sum over the 256 threads of a workgroup in a fixed order; valid in thread 0.
__device__ __forceinline__ double block_sum(double v, double *red)
{
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0)
        red[threadIdx.x >> 6] = v;
    __syncthreads();
    return ((red[0] + red[1]) + red[2]) + red[3];
}

__device__ __forceinline__ void add_sq(float g, float gs, double &acc)
{
    const float gh = gs * g;
    acc = __builtin_fma((double)gh, (double)gh, acc);   // the product of two fp32 values is exact in fp64
}

// Workgroup b sums the squares of piece b of this launch: elements [p*kPiece, (p+1)*kPiece) of
// the tensor that piece falls into, clipped to the tensor.
template <bool BF16>
__global__ __launch_bounds__(kBlock) void k_noalloc_partials(Batch bt, float gs, double *__restrict__ out)
{
    __shared__ double red[kBlock / 64];
    const int b = blockIdx.x;
    int d = 0;
    while (d + 1 < bt.count && bt.first_piece[d + 1] <= b)
        ++d;
    const int64_t e0 = (int64_t)(b - bt.first_piece[d]) * kPiece;
    const int64_t left = bt.numel[d] - e0;
    const uint32_t n = left < kPiece ? (uint32_t)left : (uint32_t)kPiece;
    const uint32_t tid = threadIdx.x;
    double acc = 0.0;
    if (BF16) {
        const uint16_t *g = static_cast<const uint16_t *>(bt.ptr[d]) + e0;
        if ((reinterpret_cast<uintptr_t>(g) & 7u) == 0) {
            const u32x2 *g4 = reinterpret_cast<const u32x2 *>(g);
            const uint32_t nvec = n / 4;
            for (uint32_t i = tid; i < nvec; i += kBlock) {
                const u32x2 v = g4[i];
                add_sq(__uint_as_float(v.x << 16), gs, acc);
                add_sq(__uint_as_float(v.x & 0xffff0000u), gs, acc);
                add_sq(__uint_as_float(v.y << 16), gs, acc);
                add_sq(__uint_as_float(v.y & 0xffff0000u), gs, acc);
            }
            for (uint32_t i = nvec * 4 + tid; i < n; i += kBlock)
                add_sq(__uint_as_float((uint32_t)g[i] << 16), gs, acc);
        } else {
            for (uint32_t i = tid; i < n; i += kBlock)
                add_sq(__uint_as_float((uint32_t)g[i] << 16), gs, acc);
        }
    } else {
        const float *g = static_cast<const float *>(bt.ptr[d]) + e0;
        if ((reinterpret_cast<uintptr_t>(g) & 15u) == 0) {
            const f32x4 *g4 = reinterpret_cast<const f32x4 *>(g);
            const uint32_t nvec = n / 4;
            for (uint32_t i = tid; i < nvec; i += kBlock) {
                const f32x4 v = g4[i];
                add_sq(v.x, gs, acc);
                add_sq(v.y, gs, acc);
                add_sq(v.z, gs, acc);
                add_sq(v.w, gs, acc);
            }
            for (uint32_t i = nvec * 4 + tid; i < n; i += kBlock)
                add_sq(g[i], gs, acc);
        } else {
            for (uint32_t i = tid; i < n; i += kBlock)
                add_sq(g[i], gs, acc);
        }
    }
    const double s = block_sum(acc, red);
    if (tid == 0)
        out[bt.slot0 + b] = s;
}

// Workgroup k adds worker k's partial sums (thread-strided, then the fixed block order) into x[k].
__global__ __launch_bounds__(kBlock) void k_noalloc_final(Ranges rg, const double *__restrict__ part,
                                                          double *__restrict__ x)
{
    __shared__ double red[kBlock / 64];
    const int k = blockIdx.x;
    double acc = 0.0;
    for (int i = rg.begin[k] + (int)threadIdx.x; i < rg.begin[k + 1]; i += kBlock)
        acc += part[i];
    const double s = block_sum(acc, red);
    if (threadIdx.x == 0)
        x[k] = s;
}

// The device address of `scratch` on each GPU, looked up once per device (the array's name
// is only a host-side stand-in; kernels must be given this address).
std::mutex g_lock;
double *g_scratch[kMaxDevices];

int32_t scratch_for_current_device(double **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess)
        return SELSYNC_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices)
        return SELSYNC_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return SELSYNC_ERR_HIP;
        }
        g_scratch[dev] = static_cast<double *>(p);
    }
    *out = g_scratch[dev];
    return SELSYNC_OK;
}

// [p, p + bytes) must be device memory of GPU `dev`, inside one allocation.
int32_t check_device_range(const void *p, size_t bytes, int dev)
{
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
        (void)hipGetLastError();
        return SELSYNC_ERR_NOT_DEVICE_MEM;
    }
    if (attr.type != hipMemoryTypeDevice || attr.device != dev)
        return SELSYNC_ERR_NOT_DEVICE_MEM;
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    if (hipMemGetAddressRange(&base, &size, const_cast<void *>(p)) != hipSuccess) {
        (void)hipGetLastError();
        return SELSYNC_ERR_NOT_DEVICE_MEM;     // no allocation known around it: nothing to check the size against
    }
    const uintptr_t lo = reinterpret_cast<uintptr_t>(p), b0 = reinterpret_cast<uintptr_t>(base);
    if (lo < b0 || lo + bytes > b0 + size)
        return SELSYNC_ERR_INVALID_ARG;
    return SELSYNC_OK;
}

}  // namespace

extern "C" int32_t selsync_grad_norm_sq_noalloc(const selsync_tensor_list *grads, int32_t num_workers,
                                                float grad_scale, double *norm_sq_out, void *stream)
{
    if (!grads || !norm_sq_out)
        return SELSYNC_ERR_INVALID_ARG;
    if (num_workers < 1)
        return SELSYNC_ERR_INVALID_ARG;
    if (num_workers > kMaxWorkersNoAlloc)
        return SELSYNC_ERR_TOO_LARGE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess)
        return SELSYNC_ERR_HIP;

    // pass 1: validate everything and count pieces before anything is enqueued
    const int T = grads[0].count;
    int32_t dtype = SELSYNC_F32;
    int64_t pieces = 0;
    for (int k = 0; k < num_workers; ++k) {
        if (grads[k].count != T || T < 0)
            return SELSYNC_ERR_SHAPE_MISMATCH;
        if (T > 0 && !grads[k].tensors)
            return SELSYNC_ERR_INVALID_ARG;
        for (int t = 0; t < T; ++t) {
            const selsync_tensor &x = grads[k].tensors[t];
            if (x.dtype != SELSYNC_F32 && x.dtype != SELSYNC_BF16)
                return SELSYNC_ERR_DTYPE;
            if (k == 0 && t == 0)
                dtype = x.dtype;
            if (x.dtype != dtype)
                return SELSYNC_ERR_DTYPE;
            if (x.numel < 0)
                return SELSYNC_ERR_INVALID_ARG;
            if (x.numel != grads[0].tensors[t].numel)
                return SELSYNC_ERR_SHAPE_MISMATCH;
            if (x.numel == 0)
                continue;
            const size_t es = x.dtype == SELSYNC_BF16 ? 2 : 4;
            if (!x.data || reinterpret_cast<uintptr_t>(x.data) % es != 0)
                return SELSYNC_ERR_INVALID_ARG;
            const int32_t rc = check_device_range(x.data, (size_t)x.numel * es, dev);
            if (rc)
                return rc;
            pieces += (x.numel + kPiece - 1) / kPiece;
            if (pieces > kMaxPieces)
                return SELSYNC_ERR_TOO_LARGE;
        }
    }
    {
        const int32_t rc = check_device_range(norm_sq_out, sizeof(double) * (size_t)num_workers, dev);
        if (rc)
            return rc;
    }
    double *part = nullptr;
    {
        const int32_t rc = scratch_for_current_device(&part);
        if (rc)
            return rc;
    }

    // pass 2: one launch per kBatch non-empty tensors, worker by worker, then the final pass
    hipStream_t s = static_cast<hipStream_t>(stream);
    Ranges rg;
    Batch bt;
    bt.count = 0;
    bt.slot0 = 0;
    bt.first_piece[0] = 0;
    int32_t slot = 0;
    auto flush = [&]() -> hipError_t {
        if (bt.count == 0)
            return hipSuccess;
        const int n = bt.first_piece[bt.count];
        if (dtype == SELSYNC_BF16)
            hipLaunchKernelGGL(k_noalloc_partials<true>, dim3(n), dim3(kBlock), 0, s, bt, grad_scale, part);
        else
            hipLaunchKernelGGL(k_noalloc_partials<false>, dim3(n), dim3(kBlock), 0, s, bt, grad_scale, part);
        bt.count = 0;
        bt.slot0 = slot;
        return hipGetLastError();
    };
    for (int k = 0; k < num_workers; ++k) {
        rg.begin[k] = slot;
        for (int t = 0; t < T; ++t) {
            const selsync_tensor &x = grads[k].tensors[t];
            if (x.numel == 0)
                continue;
            const int32_t np = (int32_t)((x.numel + kPiece - 1) / kPiece);
            bt.ptr[bt.count] = x.data;
            bt.numel[bt.count] = x.numel;
            bt.first_piece[bt.count + 1] = bt.first_piece[bt.count] + np;
            bt.count += 1;
            slot += np;
            if (bt.count == kBatch && flush() != hipSuccess)
                return SELSYNC_ERR_HIP;
        }
    }
    rg.begin[num_workers] = slot;
    if (flush() != hipSuccess)
        return SELSYNC_ERR_HIP;
    hipLaunchKernelGGL(k_noalloc_final, dim3(num_workers), dim3(kBlock), 0, s, rg, part, norm_sq_out);
    if (hipGetLastError() != hipSuccess)
        return SELSYNC_ERR_HIP;
    return SELSYNC_OK;
}
