/*
 * gfx950 encoder of the L3 format: interleaved 8-bit RGB in device memory ->
 * L3 files in device memory, byte for byte what l3_encode_cpu produces.
 *
 * arxiv 2208.08711, Section 4.2, encoding direction: per patch and channel, the
 * custom Paeth filter (rows after the first: pixel minus the nearest of the three
 * upper neighbours to TL + TR - T, taken from the ORIGINAL row above, so every
 * pixel of the patch is independent), then row-wise base-delta (row minimum as
 * base, minimal width, deltas packed).  Section 4.3: patches concatenated, their
 * offsets recorded in three arrays behind a 13-byte header.
 *
 * Three kernels per call:
 *   measure  one wave per (patch, channel): row widths -> patch byte size;
 *   layout   one workgroup per image: exclusive prefix sum of the patch sizes ->
 *            header, offset arrays, file length (this is where a scan belongs: the
 *            addends are all known);
 *   pack     one wave per (patch, channel): rows again, bits assembled in LDS with
 *            atomic OR (a row's position is the running sum of the rows before
 *            it), then copied to the file.
 * The forward filter needs no row recurrence, so a wave just walks the rows with
 * the row above in registers and lane shifts for the neighbours.
 */
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <cstring>
#include <new>

#include "l3_ctx.h"

namespace {

constexpr int kMaxPatch = 128;                       /* two pixels per lane */

struct L3EncodeDesc {
    const uint8_t* rgb;
    uint8_t* file;
    uint64_t row_stride;
    uint64_t file_cap;
    uint32_t width, height;
    uint32_t tiles_x, tiles_y;
    uint32_t patch;
    uint32_t sizes_base;     /* first entry of this image in the sizes scratch */
    uint32_t status_index;
    uint32_t pad_;
};

typedef __attribute__((address_space(1))) uint32_t global_u32_unaligned __attribute__((aligned(1)));

__device__ __forceinline__ int nearest_upper(int tl, int t, int tr) {
    /* distances to TL + TR - T: |TR - T| for TL, |TL - T| for TR, |TL + TR - 2T| for T;
     * ties: TL, then TR, then T */
    const int d_tl = abs(tr - t), d_tr = abs(tl - t), d_t = abs(tl + tr - 2 * t);
    if (d_tl <= d_tr && d_tl <= d_t) return tl;
    return d_tr <= d_t ? tr : t;
}

__device__ __forceinline__ int wave_min(int v) {
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v = min(v, __shfl_xor(v, s));
    return v;
}
__device__ __forceinline__ int wave_max(int v) {
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v = max(v, __shfl_xor(v, s));
    return v;
}

/* Walks the rows of patch (c, ty, tx).  PACK = false: returns the patch's size in
 * bits.  PACK = true: also ORs every field into `bits` (LDS, zeroed by the caller). */
template <bool PACK>
__device__ uint32_t walk_patch(const L3EncodeDesc& d, uint32_t c, uint32_t tx, uint32_t ty,
                               uint32_t* bits) {
    const uint32_t lane = threadIdx.x;
    const uint32_t n = d.patch;
    const uint32_t x0 = tx * n, y0 = ty * n;
    const uint32_t pw = min(n, d.width - x0), ph = min(n, d.height - y0);
    const bool has0 = lane < pw, has1 = lane + 64 < pw;          /* pixels lane and lane + 64 */
    const uint8_t* src = d.rgb + (size_t)y0 * d.row_stride + (size_t)x0 * 3 + c;

    int up0 = 0, up1 = 0;           /* the original row above */
    uint32_t pos = 0;               /* bit position of the current row's record */
    int next0 = has0 ? src[3 * (size_t)lane] : 0;             /* the row after, already travelling */
    int next1 = has1 ? src[3 * (size_t)(lane + 64)] : 0;
    for (uint32_t r = 0; r < ph; ++r) {
        const int cur0 = next0, cur1 = next1;
        if (r + 1 < ph) {
            const uint8_t* row = src + (size_t)(r + 1) * d.row_stride;
            next0 = has0 ? row[3 * (size_t)lane] : 0;
            next1 = has1 ? row[3 * (size_t)(lane + 64)] : 0;
        }
        int v0, v1;
        if (r == 0) {
            v0 = cur0;              /* first row raw, taken as unsigned */
            v1 = cur1;
        } else {
            /* neighbours of pixel `lane`: lanes -1/+1; of pixel `lane + 64`: the same
             * lanes' second pixels, with lanes 63 and 0 joining the halves */
            const int l0 = __shfl_up(up0, 1), r0 = __shfl_down(up0, 1);
            const int l1 = __shfl_up(up1, 1), r1 = __shfl_down(up1, 1);
            const int first1 = __shfl(up1, 0), last0 = __shfl(up0, 63);
            const int tl0 = l0, tr0 = lane == 63 ? first1 : r0;
            const int tl1 = lane == 0 ? last0 : l1, tr1 = r1;
            const bool edge0 = lane == 0 || lane + 1 == pw;
            const bool edge1 = lane + 64 + 1 == pw;
            const int p0 = edge0 ? up0 : nearest_upper(tl0, up0, tr0);
            const int p1 = edge1 ? up1 : nearest_upper(tl1, up1, tr1);
            v0 = (int)(int8_t)(uint8_t)(cur0 - p0);   /* later rows taken as signed bytes */
            v1 = (int)(int8_t)(uint8_t)(cur1 - p1);
        }
        int lo = 1 << 20, hi = -(1 << 20);
        if (has0) { lo = v0; hi = v0; }
        if (has1) { lo = min(lo, v1); hi = max(hi, v1); }
        lo = wave_min(lo);
        hi = wave_max(hi);
        const uint32_t range = (uint32_t)(hi - lo);
        const uint32_t width = range ? 32u - (uint32_t)__builtin_clz(range) : 0u;
        if (PACK) {
            if (lane == 0) {
                const uint32_t rec = width | (((uint32_t)lo & 0xFFu) << 4);
                const uint32_t sh = pos & 31u;
                atomicOr(&bits[pos >> 5], rec << sh);
                if (sh > 20) atomicOr(&bits[(pos >> 5) + 1], rec >> (32u - sh));
            }
            if (width) {
                if (has0) {
                    const uint32_t b = pos + 12 + lane * width, sh = b & 31u;
                    const uint32_t dlt = (uint32_t)(v0 - lo);
                    atomicOr(&bits[b >> 5], dlt << sh);
                    if (sh + width > 32) atomicOr(&bits[(b >> 5) + 1], dlt >> (32u - sh));
                }
                if (has1) {
                    const uint32_t b = pos + 12 + (lane + 64) * width, sh = b & 31u;
                    const uint32_t dlt = (uint32_t)(v1 - lo);
                    atomicOr(&bits[b >> 5], dlt << sh);
                    if (sh + width > 32) atomicOr(&bits[(b >> 5) + 1], dlt >> (32u - sh));
                }
            }
        }
        pos += 12 + pw * width;
        up0 = cur0;
        up1 = cur1;
    }
    return pos;
}

__global__ __launch_bounds__(64) void l3_encode_measure_kernel(const L3EncodeDesc* __restrict__ descs,
                                                               uint32_t* __restrict__ sizes) {
    const L3EncodeDesc& d = descs[blockIdx.y];
    const uint32_t patches = d.tiles_x * d.tiles_y;
    const uint32_t k = blockIdx.x;
    if (k >= 3 * patches) return;
    const uint32_t c = k / patches, i = k - c * patches;
    const uint32_t bits = walk_patch<false>(d, c, i % d.tiles_x, i / d.tiles_x, nullptr);
    if (threadIdx.x == 0) sizes[d.sizes_base + k] = (bits + 7) / 8;
}

/* One workgroup per image: offsets = exclusive prefix sum of the patch sizes. */
__global__ __launch_bounds__(256) void l3_encode_layout_kernel(const L3EncodeDesc* __restrict__ descs,
                                                               const uint32_t* __restrict__ sizes,
                                                               uint64_t* __restrict__ file_len,
                                                               uint32_t* __restrict__ status) {
    const L3EncodeDesc& d = descs[blockIdx.x];
    const uint32_t patches = d.tiles_x * d.tiles_y, total = 3 * patches;
    const uint64_t header = 13 + 12ull * patches;
    const bool header_fits = header <= d.file_cap;
    __shared__ uint64_t scan[256];
    __shared__ uint64_t carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (uint32_t first = 0; first < total; first += 256) {
        const uint32_t k = first + threadIdx.x;
        const uint64_t mine = k < total ? sizes[d.sizes_base + k] : 0;
        scan[threadIdx.x] = mine;
        __syncthreads();
        for (uint32_t step = 1; step < 256; step <<= 1) {       /* inclusive scan of the chunk */
            const uint64_t add = threadIdx.x >= step ? scan[threadIdx.x - step] : 0;
            __syncthreads();
            scan[threadIdx.x] += add;
            __syncthreads();
        }
        const uint64_t offset = carry + scan[threadIdx.x] - mine;
        if (k < total && header_fits && offset <= 0xFFFFFFFFull)
            *reinterpret_cast<global_u32_unaligned*>((uintptr_t)(d.file + 13 + 4 * (size_t)k)) = (uint32_t)offset;
        __syncthreads();
        if (threadIdx.x == 255) carry += scan[255];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const uint64_t need = header + carry;
        file_len[d.status_index] = need;
        uint32_t st = 0;
        if (need > d.file_cap) st |= 1u;                 /* output capacity too small: nothing packed */
        if (carry > 0xFFFFFFFFull) st |= 2u;             /* data section beyond 32-bit offsets */
        if (status) status[d.status_index] = st;
        if (header_fits) {
            uint8_t* f = d.file;
            f[0] = 0x4C; f[1] = 0x33; f[2] = 0x00; f[3] = 0x01;
            for (int b = 0; b < 4; ++b) {
                f[4 + b] = (uint8_t)(d.width >> (8 * b));
                f[8 + b] = (uint8_t)(d.height >> (8 * b));
            }
            f[12] = (uint8_t)d.patch;
        }
    }
}

__global__ __launch_bounds__(64) void l3_encode_pack_kernel(const L3EncodeDesc* __restrict__ descs,
                                                            const uint32_t* __restrict__ sizes,
                                                            const uint64_t* __restrict__ file_len) {
    const L3EncodeDesc& d = descs[blockIdx.y];
    const uint32_t patches = d.tiles_x * d.tiles_y;
    const uint32_t k = blockIdx.x;
    if (k >= 3 * patches) return;
    const uint64_t need = file_len[d.status_index];
    if (need > d.file_cap || need - (13 + 12ull * patches) > 0xFFFFFFFFull) return;

    extern __shared__ uint32_t bits[];   /* sized by the host for the largest patch of the launch */
    const uint32_t bytes = sizes[d.sizes_base + k];
    const uint32_t words = (bytes + 3) / 4 + 1;
    for (uint32_t i = threadIdx.x; i < words; i += 64) bits[i] = 0;
    __syncthreads();
    const uint32_t c = k / patches, i = k - c * patches;
    (void)walk_patch<true>(d, c, i % d.tiles_x, i / d.tiles_x, bits);
    __syncthreads();

    const uint32_t offset = *reinterpret_cast<const global_u32_unaligned*>((uintptr_t)(d.file + 13 + 4 * (size_t)k));
    uint8_t* dst = d.file + 13 + 12 * (size_t)patches + offset;
    const uint32_t whole = bytes / 4;
    for (uint32_t w = threadIdx.x; w < whole; w += 64)
        *reinterpret_cast<global_u32_unaligned*>((uintptr_t)(dst + 4 * (size_t)w)) = bits[w];
    const uint32_t tail = bytes - 4 * whole;
    if (threadIdx.x < tail) dst[4 * (size_t)whole + threadIdx.x] = (uint8_t)(bits[whole] >> (8 * threadIdx.x));
}

}  // namespace

/* Workspace of l3_encode_batch: descriptor table (pinned + device) and patch sizes. */
struct L3EncodeState {
    L3EncodeDesc* h_descs = nullptr;
    L3EncodeDesc* d_descs = nullptr;
    size_t desc_cap = 0;
    uint32_t* d_sizes = nullptr;
    size_t sizes_cap = 0;
    hipEvent_t done = nullptr;
    bool pending = false;
};

void l3_encode_state_free(L3EncodeState* s) {
    if (!s) return;
    if (s->pending) (void)hipEventSynchronize(s->done);
    if (s->done) (void)hipEventDestroy(s->done);
    if (s->h_descs) (void)hipHostFree(s->h_descs);
    if (s->d_descs) (void)hipFree(s->d_descs);
    if (s->d_sizes) (void)hipFree(s->d_sizes);
    delete s;
}

extern "C" l3_status l3_encode_batch(l3_ctx* ctx, const l3_encode_item* items, int n,
                                     uint64_t* d_file_len, uint32_t* d_status, void* stream_v) {
    if (!ctx || n < 0 || (n > 0 && (!items || !d_file_len))) return L3_ERR_INVALID_ARG;
    if (n == 0) return L3_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return L3_ERR_DEVICE;

    size_t total_patches = 0;
    uint32_t max_patches = 0, max_n = 1;
    for (int i = 0; i < n; ++i) {
        const l3_encode_item& it = items[i];
        if (!it.d_rgb || !it.d_file || it.width == 0 || it.height == 0 ||
            it.row_stride < (size_t)it.width * 3)
            return L3_ERR_INVALID_ARG;
        const uint32_t np = it.patch ? it.patch : l3_default_patch(it.width, it.height);
        if (np > kMaxPatch) return L3_ERR_UNSUPPORTED;
        if (np > max_n) max_n = np;
        if (it.width > (1u << 24) || it.height > (1u << 24)) return L3_ERR_UNSUPPORTED;
        const uint64_t p = (uint64_t)((it.width + np - 1) / np) * ((it.height + np - 1) / np);
        if (3 * p > 0x7FFFFFFFull) return L3_ERR_UNSUPPORTED;
        total_patches += (size_t)(3 * p);
        if (3 * p > max_patches) max_patches = (uint32_t)(3 * p);
    }
    if (total_patches > 0xFFFFFFFFull) return L3_ERR_UNSUPPORTED;

    if (!ctx->enc) {
        ctx->enc = new (std::nothrow) L3EncodeState;
        if (!ctx->enc) return L3_ERR_DEVICE;
        if (hipEventCreateWithFlags(&ctx->enc->done, hipEventDisableTiming) != hipSuccess) return L3_ERR_DEVICE;
    }
    L3EncodeState* st = ctx->enc;
    if (st->pending) {   /* the workspace is reused: wait for the previous call's kernels */
        if (hipEventSynchronize(st->done) != hipSuccess) return L3_ERR_DEVICE;
        st->pending = false;
    }
    if ((size_t)n > st->desc_cap) {
        size_t cap = 64;
        while (cap < (size_t)n) cap *= 2;
        if (st->h_descs) (void)hipHostFree(st->h_descs);
        if (st->d_descs) (void)hipFree(st->d_descs);
        st->h_descs = nullptr;
        st->d_descs = nullptr;
        st->desc_cap = 0;
        if (hipHostMalloc(reinterpret_cast<void**>(&st->h_descs), cap * sizeof(L3EncodeDesc),
                          hipHostMallocDefault) != hipSuccess ||
            hipMalloc(reinterpret_cast<void**>(&st->d_descs), cap * sizeof(L3EncodeDesc)) != hipSuccess)
            return L3_ERR_DEVICE;
        st->desc_cap = cap;
    }
    if (total_patches > st->sizes_cap) {
        size_t cap = 4096;
        while (cap < total_patches) cap *= 2;
        if (st->d_sizes) (void)hipFree(st->d_sizes);
        st->d_sizes = nullptr;
        st->sizes_cap = 0;
        if (hipMalloc(reinterpret_cast<void**>(&st->d_sizes), cap * sizeof(uint32_t)) != hipSuccess)
            return L3_ERR_DEVICE;
        st->sizes_cap = cap;
    }

    size_t base = 0;
    for (int i = 0; i < n; ++i) {
        const l3_encode_item& it = items[i];
        L3EncodeDesc& d = st->h_descs[i];
        const uint32_t np = it.patch ? it.patch : l3_default_patch(it.width, it.height);
        d.rgb = it.d_rgb;
        d.file = it.d_file;
        d.row_stride = it.row_stride;
        d.file_cap = it.file_cap;
        d.width = it.width;
        d.height = it.height;
        d.tiles_x = (it.width + np - 1) / np;
        d.tiles_y = (it.height + np - 1) / np;
        d.patch = np;
        d.sizes_base = (uint32_t)base;
        d.status_index = (uint32_t)i;
        d.pad_ = 0;
        base += 3 * (size_t)d.tiles_x * d.tiles_y;
    }
    if (hipMemcpyAsync(st->d_descs, st->h_descs, (size_t)n * sizeof(L3EncodeDesc), hipMemcpyHostToDevice,
                       stream) != hipSuccess)
        return L3_ERR_DEVICE;
    for (int first = 0; first < n; first += 65535) {
        const int m = n - first < 65535 ? n - first : 65535;
        hipLaunchKernelGGL(l3_encode_measure_kernel, dim3(max_patches, (uint32_t)m), dim3(64), 0, stream,
                           st->d_descs + first, st->d_sizes);
    }
    hipLaunchKernelGGL(l3_encode_layout_kernel, dim3((uint32_t)n), dim3(256), 0, stream, st->d_descs,
                       st->d_sizes, d_file_len, d_status);
    const size_t lds_bytes = ((size_t)max_n * (12 + 8 * (size_t)max_n) + 31) / 32 * 4 + 8;
    for (int first = 0; first < n; first += 65535) {
        const int m = n - first < 65535 ? n - first : 65535;
        hipLaunchKernelGGL(l3_encode_pack_kernel, dim3(max_patches, (uint32_t)m), dim3(64), lds_bytes,
                           stream, st->d_descs + first, st->d_sizes, d_file_len);
    }
    if (hipGetLastError() != hipSuccess) return L3_ERR_DEVICE;
    if (hipEventRecord(st->done, stream) != hipSuccess) return L3_ERR_DEVICE;
    st->pending = true;
    return L3_OK;
}
