// lagom_comm_kernel: the local data-movement step of a chunked collective on gfx950.
//
// Mapping of the paper's three resource parameters (Sec. 2.2, Sec. 3.2) onto CDNA4:
//   NC  channels   -> workgroups of the launch (each occupies wave slots of one CU),
//   NT  threads    -> workgroup size (NT/64 wavefronts),
//   C   chunk size -> the unit of work a channel takes at a time: chunk g of the byte
//                     range is moved by workgroup g mod NC.
// Inside a chunk every lane moves 16-byte vectors; consecutive lanes touch consecutive
// vectors, so one wavefront instruction covers 1 KiB of contiguous HBM.  A lane issues the
// loads of U vectors of every source before it uses any of them.  Every byte is touched
// once, so stores always carry the non-temporal hint (measured on MI355X: +3..7 % and no
// write-allocate traffic in the L2 that a co-running GEMM depends on).  Loads carry it only
// when the launch has at least kStreamLoadsFromNC channels: with that many channels the
// kernel is bandwidth-bound and streams from HBM (+6..13 %), while with few channels it is
// latency-bound and its sources are usually still in the last-level cache, where the hint
// costs 15..30 %.
//
// Arithmetic (reduce-copy): fp32 additions in source order, bf16 widened exactly by a
// 16-bit shift, one round-to-nearest-even at the store.  Only additions are used, so no
// fused operation can change the rounding.
#include <hip/hip_runtime.h>
#include <atomic>
#include "common.h"

namespace {

struct CommArgs {
    const char* src[LAGOM_MAX_SRCS];
    char* dst[LAGOM_MAX_DSTS];
    int32_t nsrc, ndst;
    int64_t shard_bytes;       // bytes per source
    int64_t chunk_bytes;       // C
    int64_t chunks_per_shard;
    int64_t total_chunks;      // reduce: chunks_per_shard; gather: nsrc * chunks_per_shard
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kStreamLoadsFromNC = 128;

template <bool STREAM>
__device__ __forceinline__ u32x4 ld16(const char* p) {
    if (STREAM) return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return *reinterpret_cast<const u32x4*>(p);
}
__device__ __forceinline__ void st16(char* p, u32x4 v) { __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p)); }

// bf16 is the upper half of an fp32 pattern.
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest, ties to even; NaN keeps a quiet payload.
__device__ __forceinline__ uint32_t bf16_round(float f) {
    const uint32_t u = __float_as_uint(f);
    const uint32_t upper = u >> 16, lower = u & 0xffffu;
    const uint32_t up = (lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) ? 1u : 0u;
    const uint32_t r = upper + up;
    return ((u & 0x7fffffffu) > 0x7f800000u) ? (upper | 0x0040u) : r;
}

template <int DT>
struct Acc;

// fp32: one 16-byte vector = 4 elements
template <>
struct Acc<LAGOM_F32> {
    f32x4 a;
    __device__ __forceinline__ void init(u32x4 v) { a = __builtin_bit_cast(f32x4, v); }
    __device__ __forceinline__ void add(u32x4 v) { a = a + __builtin_bit_cast(f32x4, v); }
    __device__ __forceinline__ u32x4 result() const { return __builtin_bit_cast(u32x4, a); }
};

// bf16: one 16-byte vector = 8 elements, accumulated as 8 fp32
template <>
struct Acc<LAGOM_BF16> {
    float a[8];
    __device__ __forceinline__ void init(u32x4 v) {
#pragma unroll
        for (int i = 0; i < 4; ++i) { a[2 * i] = bf16_lo(v[i]); a[2 * i + 1] = bf16_hi(v[i]); }
    }
    __device__ __forceinline__ void add(u32x4 v) {
#pragma unroll
        for (int i = 0; i < 4; ++i) { a[2 * i] = a[2 * i] + bf16_lo(v[i]); a[2 * i + 1] = a[2 * i + 1] + bf16_hi(v[i]); }
    }
    __device__ __forceinline__ u32x4 result() const {
        u32x4 r;
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = bf16_round(a[2 * i]) | (bf16_round(a[2 * i + 1]) << 16);
        return r;
    }
};

// One element of a short tail (fewer than 16 bytes left at the end of the buffer).
template <int DT, class SRC, class DST>
__device__ __forceinline__ void reduce_tail_element(const SRC& src, const DST& dst, int nsrc, int ndst, int64_t byte_off) {
    if (DT == LAGOM_F32) {
        float acc = *reinterpret_cast<const float*>(src(0) + byte_off);
        for (int s = 1; s < nsrc; ++s) acc = acc + *reinterpret_cast<const float*>(src(s) + byte_off);
        for (int d = 0; d < ndst; ++d) *reinterpret_cast<float*>(dst(d) + byte_off) = acc;
    } else {
        float acc = bf16_lo(*reinterpret_cast<const uint16_t*>(src(0) + byte_off));
        for (int s = 1; s < nsrc; ++s) acc = acc + bf16_lo(*reinterpret_cast<const uint16_t*>(src(s) + byte_off));
        const uint16_t r = (uint16_t)bf16_round(acc);
        for (int d = 0; d < ndst; ++d) *reinterpret_cast<uint16_t*>(dst(d) + byte_off) = r;
    }
}

// One chunk [base, base + len) of a reduce-copy, moved by the nt threads of a workgroup.
// S > 0: number of sources known at compile time (all loads of a batch issued before the
// first add).  S == 0: any number of sources, loaded source by source.
// U: 16-byte vectors a lane has in flight per source.  src(s) / dst(d) give the buffers.
template <int DT, int S, int U, bool STREAM, class SRC, class DST>
__device__ __forceinline__ void reduce_chunk(const SRC& src, const DST& dst, int nsrc, int ndst, int64_t base, int64_t len, int tid, int nt) {
    const int esize = DT == LAGOM_F32 ? 4 : 2;
    const int64_t nvec = len >> 4;
    int64_t v = tid;
    if constexpr (S > 0) {
        // full batches: U vectors per source per lane, strided by the workgroup size
        for (; v + (int64_t)(U - 1) * nt < nvec; v += (int64_t)U * nt) {
            u32x4 r[S][U];
#pragma unroll
            for (int s = 0; s < S; ++s)
#pragma unroll
                for (int u = 0; u < U; ++u) r[s][u] = ld16<STREAM>(src(s) + base + ((v + (int64_t)u * nt) << 4));
#pragma unroll
            for (int u = 0; u < U; ++u) {
                Acc<DT> acc;
                acc.init(r[0][u]);
#pragma unroll
                for (int s = 1; s < S; ++s) acc.add(r[s][u]);
                const u32x4 o = acc.result();
                for (int d = 0; d < ndst; ++d) st16(dst(d) + base + ((v + (int64_t)u * nt) << 4), o);
            }
        }
    }
    // remaining vectors (and every vector when S == 0)
    for (; v < nvec; v += nt) {
        const int64_t off = base + (v << 4);
        Acc<DT> acc;
        acc.init(ld16<STREAM>(src(0) + off));
        const int ns = S > 0 ? S : nsrc;
        int s = 1;
        for (; s + 3 < ns; s += 4) {          // four loads in flight, added in source order
            const u32x4 x0 = ld16<STREAM>(src(s) + off), x1 = ld16<STREAM>(src(s + 1) + off);
            const u32x4 x2 = ld16<STREAM>(src(s + 2) + off), x3 = ld16<STREAM>(src(s + 3) + off);
            acc.add(x0); acc.add(x1); acc.add(x2); acc.add(x3);
        }
        for (; s < ns; ++s) acc.add(ld16<STREAM>(src(s) + off));
        const u32x4 o = acc.result();
        for (int d = 0; d < ndst; ++d) st16(dst(d) + off, o);
    }
    // fewer than 16 bytes at the very end of the buffer
    const int tail_elems = (int)(len & 15) / esize;
    if (tid < tail_elems) reduce_tail_element<DT>(src, dst, nsrc, ndst, base + (nvec << 4) + (int64_t)tid * esize);
}

// One chunk of a plain copy of one source to ndst destinations (bytes are moved, never interpreted).
template <int U, bool STREAM, class DST>
__device__ __forceinline__ void copy_chunk(const char* src, const DST& dst, int ndst, int64_t dst_off, int64_t len, int tid, int nt) {
    const int64_t nvec = len >> 4;
    int64_t v = tid;
    for (; v + (int64_t)(U - 1) * nt < nvec; v += (int64_t)U * nt) {
        u32x4 x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = ld16<STREAM>(src + ((v + (int64_t)u * nt) << 4));
#pragma unroll
        for (int u = 0; u < U; ++u)
            for (int d = 0; d < ndst; ++d) st16(dst(d) + dst_off + ((v + (int64_t)u * nt) << 4), x[u]);
    }
    for (; v < nvec; v += nt) {
        const u32x4 x = ld16<STREAM>(src + (v << 4));
        for (int d = 0; d < ndst; ++d) st16(dst(d) + dst_off + (v << 4), x);
    }
    const int tail = (int)(len & 15);          // only at the very end of a buffer: bytes, copied one by one
    if (tid < tail) {
        const char b = src[(nvec << 4) + tid];
        for (int d = 0; d < ndst; ++d) dst(d)[dst_off + (nvec << 4) + tid] = b;
    }
}

template <int DT, int S, int U, bool STREAM, int MAXNT>
__global__ void __launch_bounds__(MAXNT) reduce_copy_kernel(const CommArgs p) {
    const auto src = [&p](int s) { return p.src[s]; };
    const auto dst = [&p](int d) { return p.dst[d]; };
    for (int64_t g = blockIdx.x; g < p.total_chunks; g += gridDim.x) {
        const int64_t base = g * p.chunk_bytes;
        const int64_t left = p.shard_bytes - base;
        reduce_chunk<DT, S, U, STREAM>(src, dst, p.nsrc, p.ndst, base, left < p.chunk_bytes ? left : p.chunk_bytes, threadIdx.x, blockDim.x);
    }
}

// Gather-copy with 16-byte vectors; needs shard_bytes % 16 == 0 (or a single shard) so that
// every shard starts 16-byte aligned in the destination.
template <int U, bool STREAM, int MAXNT>
__global__ void __launch_bounds__(MAXNT) gather_copy_kernel(const CommArgs p) {
    const auto dst = [&p](int d) { return p.dst[d]; };
    for (int64_t g = blockIdx.x; g < p.total_chunks; g += gridDim.x) {
        const int64_t r = g / p.chunks_per_shard;
        const int64_t base = (g - r * p.chunks_per_shard) * p.chunk_bytes;
        const int64_t left = p.shard_bytes - base;
        copy_chunk<U, STREAM>(p.src[r] + base, dst, p.ndst, r * p.shard_bytes + base, left < p.chunk_bytes ? left : p.chunk_bytes,
                              threadIdx.x, blockDim.x);
    }
}

// Gather-copy for shards whose byte length is not a multiple of 16: destinations of shards
// r >= 1 are then only element-aligned, so elements (2 or 4 bytes) are copied one by one.
template <typename E>
__global__ void __launch_bounds__(1024) gather_copy_elements_kernel(const CommArgs p) {
    const int nt = blockDim.x;
    for (int64_t g = blockIdx.x; g < p.total_chunks; g += gridDim.x) {
        const int64_t r = g / p.chunks_per_shard;
        const int64_t base = (g - r * p.chunks_per_shard) * p.chunk_bytes;
        const int64_t left = p.shard_bytes - base;
        const int64_t len = left < p.chunk_bytes ? left : p.chunk_bytes;
        const int64_t n = len / (int64_t)sizeof(E);
        const E* src = reinterpret_cast<const E*>(p.src[r] + base);
        for (int64_t i = threadIdx.x; i < n; i += nt) {
            const E x = src[i];
            for (int d = 0; d < p.ndst; ++d) reinterpret_cast<E*>(p.dst[d] + r * p.shard_bytes + base)[i] = x;
        }
    }
}

// MAXNT is the launch bound the kernel is compiled for: 512 threads leave 256 registers per lane,
// 1024 only 128.  Measured on the eight-source bf16 reduce: the same code compiled for 1024 threads
// loses up to 40 % at 512 threads because the loads of a batch no longer stay in flight together.
template <int DT, bool STREAM, int MAXNT>
void launch_reduce(const CommArgs& a, dim3 grid, dim3 block, hipStream_t st) {
    switch (a.nsrc) {
        case 1: hipLaunchKernelGGL((reduce_copy_kernel<DT, 1, 4, STREAM, MAXNT>), grid, block, 0, st, a); break;
        case 2: hipLaunchKernelGGL((reduce_copy_kernel<DT, 2, 4, STREAM, MAXNT>), grid, block, 0, st, a); break;
        case 3: hipLaunchKernelGGL((reduce_copy_kernel<DT, 3, 4, STREAM, MAXNT>), grid, block, 0, st, a); break;
        case 4: hipLaunchKernelGGL((reduce_copy_kernel<DT, 4, 4, STREAM, MAXNT>), grid, block, 0, st, a); break;
        case 8: hipLaunchKernelGGL((reduce_copy_kernel<DT, 8, 2, STREAM, MAXNT>), grid, block, 0, st, a); break;
        default: hipLaunchKernelGGL((reduce_copy_kernel<DT, 0, 1, STREAM, MAXNT>), grid, block, 0, st, a); break;
    }
}

template <int DT, bool STREAM>
void launch_reduce_nt(const CommArgs& a, dim3 grid, dim3 block, hipStream_t st) {
    if (block.x <= 512) launch_reduce<DT, STREAM, 512>(a, grid, block, st);
    else launch_reduce<DT, STREAM, 1024>(a, grid, block, st);
}

template <bool STREAM>
void launch_gather(const CommArgs& a, dim3 grid, dim3 block, hipStream_t st) {
    if (block.x <= 512) hipLaunchKernelGGL((gather_copy_kernel<4, STREAM, 512>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((gather_copy_kernel<4, STREAM, 1024>), grid, block, 0, st, a);
}

// Several local steps of one collective in one launch: the channels are persistent and every channel walks the steps in
// order, taking chunks k, k+NC, ... of each (how a ring collective runs inside a collective library: one kernel whose
// channels loop over the ring steps).  Every buffer of every step holds the same number of bytes, so a given byte offset
// is always moved by the same lane of the same channel: a location that one step writes and a later step reads or
// overwrites through the same pointer is ordered by that lane's program order.  There is no synchronisation between
// channels.
constexpr int kMaxSteps = LAGOM_MAX_STEPS;
constexpr int kMaxStepPtrs = LAGOM_MAX_STEP_PTRS;
struct StepsArgs {
    const char* ptr[kMaxStepPtrs];    // per step: its sources, then its destinations
    uint16_t first[kMaxSteps];
    uint8_t nsrc[kMaxSteps], ndst[kMaxSteps], op[kMaxSteps];
    int32_t nsteps;
    int64_t bytes;                    // per buffer
    int64_t chunk_bytes, total_chunks;
};

template <int DT, int S, int U, bool STREAM>
__device__ __forceinline__ void reduce_step(const StepsArgs& p, int first, int nsrc, int ndst) {
    const auto src = [&p, first](int s) { return p.ptr[first + s]; };
    const auto dst = [&p, first, nsrc](int d) { return const_cast<char*>(p.ptr[first + nsrc + d]); };
    for (int64_t g = blockIdx.x; g < p.total_chunks; g += gridDim.x) {
        const int64_t base = g * p.chunk_bytes;
        const int64_t left = p.bytes - base;
        reduce_chunk<DT, S, U, STREAM>(src, dst, nsrc, ndst, base, left < p.chunk_bytes ? left : p.chunk_bytes, threadIdx.x, blockDim.x);
    }
}

template <int DT, bool STREAM, int MAXNT>
__global__ void __launch_bounds__(MAXNT) comm_steps_kernel(const StepsArgs p) {
    for (int st = 0; st < p.nsteps; ++st) {
        const int first = p.first[st], nsrc = p.nsrc[st], ndst = p.ndst[st];
        if (p.op[st] == LAGOM_GATHER_COPY) {        // one source: a plain copy to every destination
            const auto dst = [&p, first](int d) { return const_cast<char*>(p.ptr[first + 1 + d]); };
            for (int64_t g = blockIdx.x; g < p.total_chunks; g += gridDim.x) {
                const int64_t base = g * p.chunk_bytes;
                const int64_t left = p.bytes - base;
                copy_chunk<4, STREAM>(p.ptr[first] + base, dst, ndst, base, left < p.chunk_bytes ? left : p.chunk_bytes, threadIdx.x, blockDim.x);
            }
        } else if (nsrc == 1) {
            reduce_step<DT, 1, 4, STREAM>(p, first, nsrc, ndst);
        } else if (nsrc == 2) {
            reduce_step<DT, 2, 4, STREAM>(p, first, nsrc, ndst);
        } else {
            reduce_step<DT, 0, 1, STREAM>(p, first, nsrc, ndst);
        }
    }
}

template <int DT, bool STREAM>
void launch_steps(const StepsArgs& a, dim3 grid, dim3 block, hipStream_t st) {
    if (block.x <= 512) hipLaunchKernelGGL((comm_steps_kernel<DT, STREAM, 512>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((comm_steps_kernel<DT, STREAM, 1024>), grid, block, 0, st, a);
}

// ------------------------------------------------------------------ staged through LDS
// The same operators with every source vector staged through LDS by direct-to-LDS loads (global_load_lds, 16 bytes per
// lane), the form the brief for this build sketches.  Each wavefront owns a ring of LDS_STAGES stages of LDS_U KiB and
// treats (batch of LDS_U KiB of the chunk, source) pairs as a stream of items: the loads of the next LDS_STAGES - 1 items
// are in flight while the current one is read back (ds_read_b128) and folded into the lane's accumulators, in source
// order, so the arithmetic and its order are exactly those of the register path; after the last source the batch is
// rounded and stored.  LDS per workgroup is (NT / 64) * LDS_STAGES * LDS_U KiB whatever the number of sources.  A
// wavefront reads only what its own loads wrote and waits for them with its own vmcnt, so there are no barriers.
// What does not fill whole batches at the end of a chunk goes through the register path.
// Measured slower than the register path by 3 - 8 % alone, and a workgroup that holds LDS cannot share a compute unit with
// a GEMM workgroup (which takes all 160 KiB): kept as a selectable path, not the default.
constexpr int LDS_STAGES = 4, LDS_U = 2;                  // 8 KiB per wavefront, 128 KiB for 1024 threads
constexpr int LDS_BYTES_PER_WAVE = LDS_STAGES * LDS_U * 1024;

__device__ __forceinline__ void dma16(const char* g, u32x4* lds_wave_uniform) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                     (__attribute__((address_space(3))) void*)lds_wave_uniform, 16, 0, 0);
}

// waits until at most `younger` items issued after the wanted one are still in flight (loads complete in issue order;
// stores share the counter and can only make the wait longer)
__device__ __forceinline__ void wait_items(int younger) {
    if (younger >= 3) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(3 * LDS_U) : "memory");
    else if (younger == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LDS_U) : "memory");
    else if (younger == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LDS_U) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// GATHER: items are batches of the one source `src(0)`, copied to dst(d) + dst_off; else a reduce-copy of nsrc sources.
template <int DT, bool GATHER, class SRC, class DST>
__device__ __forceinline__ void lds_chunk(u32x4* ring, const SRC& src, const DST& dst, int nsrc, int ndst, int64_t base, int64_t dst_base,
                                          int64_t len, int lane, int wave, int nw) {
    constexpr int64_t BATCH = LDS_U * 1024;                       // bytes of one source a wavefront moves per batch
    const int64_t nbatch = len / BATCH;                           // whole batches of the chunk, dealt to the wavefronts round-robin
    const int64_t mine = nbatch > wave ? (nbatch - wave + nw - 1) / nw : 0;
    const int S = GATHER ? 1 : nsrc;
    const int64_t items = mine * S;
    auto issue = [&](int64_t i) {
        const int64_t b = i / S;
        const int s = (int)(i - b * S);
        const char* g = src(s) + base + (wave + b * nw) * BATCH + lane * 16;
        u32x4* st = ring + (i % LDS_STAGES) * (LDS_U * 64);
#pragma unroll
        for (int u = 0; u < LDS_U; ++u) dma16(g + u * 1024, st + u * 64);
    };
    int64_t issued = 0;
    for (; issued < items && issued < LDS_STAGES - 1; ++issued) issue(issued);
    Acc<DT> acc[LDS_U];
    for (int64_t i = 0; i < items; ++i) {
        if (issued < items) { issue(issued); ++issued; }
        wait_items((int)(issued - i - 1));
        const u32x4* st = ring + (i % LDS_STAGES) * (LDS_U * 64);
        const int64_t b = i / S;
        const int s = (int)(i - b * S);
        const int64_t off = (wave + b * nw) * BATCH + lane * 16;
        if (GATHER) {
#pragma unroll
            for (int u = 0; u < LDS_U; ++u) {
                const u32x4 x = st[u * 64 + lane];
                for (int d = 0; d < ndst; ++d) st16(dst(d) + dst_base + off + u * 1024, x);
            }
        } else {
#pragma unroll
            for (int u = 0; u < LDS_U; ++u) {
                const u32x4 x = st[u * 64 + lane];
                if (s == 0) acc[u].init(x); else acc[u].add(x);
            }
            if (s == S - 1) {
#pragma unroll
                for (int u = 0; u < LDS_U; ++u) {
                    const u32x4 o = acc[u].result();
                    for (int d = 0; d < ndst; ++d) st16(dst(d) + dst_base + off + u * 1024, o);
                }
            }
        }
    }
}

template <int DT, bool GATHER, int MAXNT>
__global__ void __launch_bounds__(MAXNT) comm_lds_kernel(const CommArgs p) {
    extern __shared__ u32x4 lds_ring[];
    const int tid = threadIdx.x, lane = tid & 63, nw = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    u32x4* ring = lds_ring + wave * (LDS_BYTES_PER_WAVE / 16);
    const auto dst = [&p](int d) { return p.dst[d]; };
    for (int64_t g = blockIdx.x; g < p.total_chunks; g += gridDim.x) {
        const int64_t r = GATHER ? g / p.chunks_per_shard : 0;
        const int64_t base = (g - r * p.chunks_per_shard) * p.chunk_bytes;
        const int64_t left = p.shard_bytes - base;
        const int64_t len = left < p.chunk_bytes ? left : p.chunk_bytes;
        const int64_t bulk = len / (LDS_U * 1024) * (LDS_U * 1024);
        const int64_t dst_base = r * p.shard_bytes + base;
        if (GATHER) {
            const char* one = p.src[r];
            const auto src = [one](int) { return one; };
            lds_chunk<DT, true>(ring, src, dst, 1, p.ndst, base, dst_base, len, lane, wave, nw);
            copy_chunk<1, false>(one + base + bulk, dst, p.ndst, dst_base + bulk, len - bulk, tid, blockDim.x);
        } else {
            const auto src = [&p](int s) { return p.src[s]; };
            lds_chunk<DT, false>(ring, src, dst, p.nsrc, p.ndst, base, dst_base, len, lane, wave, nw);
            reduce_chunk<DT, 0, 1, false>(src, dst, p.nsrc, p.ndst, base + bulk, len - bulk, tid, blockDim.x);
        }
    }
}

template <void (*KERNEL)(const CommArgs)>
int launch_lds(const CommArgs& a, dim3 grid, dim3 block, hipStream_t st) {
    const int lds_bytes = (int)(block.x / 64) * LDS_BYTES_PER_WAVE;
    static std::atomic<uint64_t> done_on_device{0};     // once per kernel and device; a failure is not remembered
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) dev = 63;
    const uint64_t bit = uint64_t{1} << dev;
    if (dev == 63 || !(done_on_device.load(std::memory_order_acquire) & bit)) {
        const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(KERNEL), hipFuncAttributeMaxDynamicSharedMemorySize, 16 * LDS_BYTES_PER_WAVE);
        if (attr != hipSuccess) return lagom::fail(LAGOM_EHIP, "cannot raise the LDS limit: %s", hipGetErrorString(attr));
        done_on_device.fetch_or(bit, std::memory_order_release);
    }
    hipLaunchKernelGGL(KERNEL, grid, block, lds_bytes, st, a);
    return LAGOM_OK;
}

}  // namespace

namespace lagom {

int check_cfg(const lagom_cfg* cfg) {
    if (!cfg) return fail(LAGOM_EINVAL, "null configuration");
    if (cfg->nc < 1 || cfg->nc > 65535) return fail(LAGOM_EINVAL, "nc=%d outside 1..65535", cfg->nc);
    if (cfg->nt < 64 || cfg->nt > 1024 || cfg->nt % 64) return fail(LAGOM_EINVAL, "nt=%d must be a multiple of 64 in 64..1024", cfg->nt);
    if (cfg->chunk_bytes < 16 || cfg->chunk_bytes % 16) return fail(LAGOM_EINVAL, "chunk_bytes=%lld must be a positive multiple of 16", (long long)cfg->chunk_bytes);
    return LAGOM_OK;
}

int check_comm_args(int op, int dtype, const void* const* srcs, int nsrc, void* const* dsts, int ndst, int64_t count) {
    if (op != LAGOM_REDUCE_COPY && op != LAGOM_GATHER_COPY) return fail(LAGOM_EINVAL, "unknown op %d", op);
    if (elem_size(dtype) == 0) return fail(LAGOM_EINVAL, "unknown dtype %d", dtype);
    if (!srcs || !dsts) return fail(LAGOM_EINVAL, "null pointer array");
    if (nsrc < 1 || nsrc > LAGOM_MAX_SRCS) return fail(LAGOM_EINVAL, "nsrc=%d outside 1..%d", nsrc, LAGOM_MAX_SRCS);
    if (ndst < 1 || ndst > LAGOM_MAX_DSTS) return fail(LAGOM_EINVAL, "ndst=%d outside 1..%d", ndst, LAGOM_MAX_DSTS);
    if (count < 0 || count > (int64_t)1 << 40) return fail(LAGOM_EINVAL, "count=%lld out of range", (long long)count);
    for (int s = 0; s < nsrc; ++s) {
        if (!srcs[s]) return fail(LAGOM_EINVAL, "source %d is null", s);
        if ((uintptr_t)srcs[s] & 15) return fail(LAGOM_EALIGN, "source %d is not 16-byte aligned", s);
    }
    for (int d = 0; d < ndst; ++d) {
        if (!dsts[d]) return fail(LAGOM_EINVAL, "destination %d is null", d);
        if ((uintptr_t)dsts[d] & 15) return fail(LAGOM_EALIGN, "destination %d is not 16-byte aligned", d);
    }
    return LAGOM_OK;
}

}  // namespace lagom

extern "C" int64_t lagom_comm_bytes(int op, int dtype, int nsrc, int ndst, int64_t count) {
    const int es = lagom::elem_size(dtype);
    if (es == 0 || nsrc < 1 || ndst < 1 || count < 0) return -1;
    if (op == LAGOM_REDUCE_COPY) return (int64_t)(nsrc + ndst) * count * es;
    if (op == LAGOM_GATHER_COPY) return (int64_t)(1 + ndst) * nsrc * count * es;
    return -1;
}

extern "C" int lagom_comm_kernel(lagom_op op, lagom_dtype dt, const void* const* srcs, int nsrc,
                                 void* const* dsts, int ndst, int64_t count, const lagom_cfg* cfg, void* hip_stream) {
    if (int rc = lagom::check_comm_args(op, dt, srcs, nsrc, dsts, ndst, count)) return rc;
    if (int rc = lagom::check_cfg(cfg)) return rc;
    if (count == 0) return LAGOM_OK;

    CommArgs a{};
    for (int s = 0; s < nsrc; ++s) a.src[s] = static_cast<const char*>(srcs[s]);
    for (int d = 0; d < ndst; ++d) a.dst[d] = static_cast<char*>(dsts[d]);
    a.nsrc = nsrc; a.ndst = ndst;
    a.shard_bytes = count * lagom::elem_size(dt);
    a.chunk_bytes = cfg->chunk_bytes;
    a.chunks_per_shard = (a.shard_bytes + a.chunk_bytes - 1) / a.chunk_bytes;
    a.total_chunks = op == LAGOM_REDUCE_COPY ? a.chunks_per_shard : a.chunks_per_shard * nsrc;

    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const dim3 grid((unsigned)cfg->nc), block((unsigned)cfg->nt);
    const bool stream = cfg->nc >= kStreamLoadsFromNC;
    if (op == LAGOM_REDUCE_COPY) {
        if (dt == LAGOM_F32) stream ? launch_reduce_nt<LAGOM_F32, true>(a, grid, block, st) : launch_reduce_nt<LAGOM_F32, false>(a, grid, block, st);
        else stream ? launch_reduce_nt<LAGOM_BF16, true>(a, grid, block, st) : launch_reduce_nt<LAGOM_BF16, false>(a, grid, block, st);
    } else if (nsrc == 1 || (a.shard_bytes & 15) == 0) {
        stream ? launch_gather<true>(a, grid, block, st) : launch_gather<false>(a, grid, block, st);
    } else if (dt == LAGOM_F32) {
        hipLaunchKernelGGL((gather_copy_elements_kernel<uint32_t>), grid, block, 0, st, a);
    } else {
        hipLaunchKernelGGL((gather_copy_elements_kernel<uint16_t>), grid, block, 0, st, a);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return lagom::fail(LAGOM_EHIP, "comm kernel launch: %s", hipGetErrorString(e));
    return LAGOM_OK;
}

namespace lagom {

// Shape rules of lagom_comm_steps; also used by the overlap runner before it fuses launches.
int check_comm_steps(int dtype, const lagom_comm_step* steps, int nsteps, int64_t count) {
    if (elem_size(dtype) == 0) return fail(LAGOM_EINVAL, "unknown dtype %d", dtype);
    if (!steps || nsteps < 1 || nsteps > LAGOM_MAX_STEPS) return fail(LAGOM_EINVAL, "nsteps=%d outside 1..%d", nsteps, LAGOM_MAX_STEPS);
    if (count < 0 || count > (int64_t)1 << 40) return fail(LAGOM_EINVAL, "count=%lld out of range", (long long)count);
    int nptr = 0;
    for (int i = 0; i < nsteps; ++i) {
        const lagom_comm_step& s = steps[i];
        if (int rc = check_comm_args(s.op, dtype, s.srcs, s.nsrc, s.dsts, s.ndst, count)) return rc;
        if (s.op == LAGOM_GATHER_COPY && s.nsrc != 1)
            return fail(LAGOM_EINVAL, "step %d: a gather-copy step of a fused launch forwards one source (every buffer of every step holds `count` elements)", i);
        nptr += s.nsrc + s.ndst;
    }
    if (nptr > LAGOM_MAX_STEP_PTRS) return fail(LAGOM_EINVAL, "%d buffers in all steps together, at most %d", nptr, LAGOM_MAX_STEP_PTRS);
    // two steps may touch the same memory only through the same pointer (then the same lane moves it in both);
    // buffers that overlap in part would be moved by different lanes with nothing ordering them
    const int64_t bytes = count * elem_size(dtype);
    for (int i = 0; i < nsteps; ++i)
        for (int j = i + 1; j < nsteps; ++j) {
            const lagom_comm_step &a = steps[i], &b = steps[j];
            for (int x = 0; x < a.nsrc + a.ndst; ++x)
                for (int y = 0; y < b.nsrc + b.ndst; ++y) {
                    if (x < a.nsrc && y < b.nsrc) continue;        // both only read
                    const uintptr_t pa = (uintptr_t)(x < a.nsrc ? a.srcs[x] : a.dsts[x - a.nsrc]);
                    const uintptr_t pb = (uintptr_t)(y < b.nsrc ? b.srcs[y] : b.dsts[y - b.nsrc]);
                    if (pa != pb && pa < pb + (uintptr_t)bytes && pb < pa + (uintptr_t)bytes)
                        return fail(LAGOM_EINVAL, "steps %d and %d touch buffers that overlap in part", i, j);
                }
        }
    return LAGOM_OK;
}

}  // namespace lagom

extern "C" int lagom_comm_steps(lagom_dtype dt, const lagom_comm_step* steps, int nsteps, int64_t count,
                                const lagom_cfg* cfg, void* hip_stream) {
    if (int rc = lagom::check_comm_steps(dt, steps, nsteps, count)) return rc;
    if (int rc = lagom::check_cfg(cfg)) return rc;
    if (count == 0) return LAGOM_OK;
    StepsArgs a{};
    int n = 0;
    for (int i = 0; i < nsteps; ++i) {
        a.first[i] = (uint16_t)n; a.nsrc[i] = (uint8_t)steps[i].nsrc; a.ndst[i] = (uint8_t)steps[i].ndst; a.op[i] = (uint8_t)steps[i].op;
        for (int s = 0; s < steps[i].nsrc; ++s) a.ptr[n++] = static_cast<const char*>(steps[i].srcs[s]);
        for (int d = 0; d < steps[i].ndst; ++d) a.ptr[n++] = static_cast<const char*>(steps[i].dsts[d]);
    }
    a.nsteps = nsteps;
    a.bytes = count * lagom::elem_size(dt);
    a.chunk_bytes = cfg->chunk_bytes;
    a.total_chunks = (a.bytes + a.chunk_bytes - 1) / a.chunk_bytes;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const dim3 grid((unsigned)cfg->nc), block((unsigned)cfg->nt);
    const bool stream = cfg->nc >= kStreamLoadsFromNC;
    if (dt == LAGOM_F32) stream ? launch_steps<LAGOM_F32, true>(a, grid, block, st) : launch_steps<LAGOM_F32, false>(a, grid, block, st);
    else stream ? launch_steps<LAGOM_BF16, true>(a, grid, block, st) : launch_steps<LAGOM_BF16, false>(a, grid, block, st);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return lagom::fail(LAGOM_EHIP, "comm steps launch: %s", hipGetErrorString(e));
    return LAGOM_OK;
}

extern "C" int lagom_comm_kernel_lds(lagom_op op, lagom_dtype dt, const void* const* srcs, int nsrc,
                                     void* const* dsts, int ndst, int64_t count, const lagom_cfg* cfg, void* hip_stream) {
    if (int rc = lagom::check_comm_args(op, dt, srcs, nsrc, dsts, ndst, count)) return rc;
    if (int rc = lagom::check_cfg(cfg)) return rc;
    if (count == 0) return LAGOM_OK;
    const int64_t shard_bytes = count * lagom::elem_size(dt);
    if (op == LAGOM_GATHER_COPY && nsrc > 1 && (shard_bytes & 15))     // element-aligned shards: nothing to stage 16 bytes at a time
        return lagom_comm_kernel(op, dt, srcs, nsrc, dsts, ndst, count, cfg, hip_stream);
    CommArgs a{};
    for (int s = 0; s < nsrc; ++s) a.src[s] = static_cast<const char*>(srcs[s]);
    for (int d = 0; d < ndst; ++d) a.dst[d] = static_cast<char*>(dsts[d]);
    a.nsrc = nsrc; a.ndst = ndst;
    a.shard_bytes = shard_bytes;
    a.chunk_bytes = cfg->chunk_bytes;
    a.chunks_per_shard = (a.shard_bytes + a.chunk_bytes - 1) / a.chunk_bytes;
    a.total_chunks = op == LAGOM_REDUCE_COPY ? a.chunks_per_shard : a.chunks_per_shard * nsrc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const dim3 grid((unsigned)cfg->nc), block((unsigned)cfg->nt);
    const bool small = block.x <= 512;
    int rc;
    if (op == LAGOM_GATHER_COPY) rc = small ? launch_lds<comm_lds_kernel<LAGOM_F32, true, 512>>(a, grid, block, st) : launch_lds<comm_lds_kernel<LAGOM_F32, true, 1024>>(a, grid, block, st);
    else if (dt == LAGOM_F32) rc = small ? launch_lds<comm_lds_kernel<LAGOM_F32, false, 512>>(a, grid, block, st) : launch_lds<comm_lds_kernel<LAGOM_F32, false, 1024>>(a, grid, block, st);
    else rc = small ? launch_lds<comm_lds_kernel<LAGOM_BF16, false, 512>>(a, grid, block, st) : launch_lds<comm_lds_kernel<LAGOM_BF16, false, 1024>>(a, grid, block, st);
    if (rc) return rc;
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return lagom::fail(LAGOM_EHIP, "comm kernel launch: %s", hipGetErrorString(e));
    return LAGOM_OK;
}
