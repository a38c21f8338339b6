// lagom_gemm: C[M,N] = A[M,K] . B, bf16 inputs, fp32 accumulation on the gfx950 matrix
// cores, the computation whose slow-down the overlap model describes (Sec. 3.2, Fig. 3).
//
// Tiling: one workgroup of 256 threads (4 wavefronts, 2 x 2) owns a 256 x 256 tile of C and
// walks K in steps of 64; each wavefront owns a 128 x 128 block, i.e. 256 fp32 accumulators per
// lane (the whole AGPR file), so one workgroup is resident per compute unit.  Products that at
// most 256 tiles of 128 x 128 or of 256 x 128 cover use those instead: 256 x 256 tiles would
// leave compute units idle (see the small-tile kernels below).
// Workgroup ids are remapped so that the workgroups of one XCD (ids equal modulo 8) cover a
// compact block of tiles and share A/B panels in that XCD's L2.
//
// Fast kernel (64 <= K <= 2^22; described for B stored [N,K] and K a multiple of 64):
//   * v_mfma_f32_16x16x32_bf16, 8 x 8 MFMA tiles per wavefront.  Under random operands the chip
//     is power limited, and this shape costs less energy per flop than 32x32x16: a register-only
//     loop sustains 86 % of the 2.5 PFLOP/s peak at 2.14 GHz with it against 77 % at 1.89 GHz.
//     The MFMAs are inline asm with the accumulators pinned to AGPRs (with the builtin the
//     register allocator copies the 64 accumulator quads around on every iteration).
//   * A and B tiles go from global memory straight into LDS (global_load_lds_dwordx4, scalar base
//     + 32-bit lane offset).  LDS holds five 32 KiB slots used as a ring A0,B0,A1,B1,A2,...: while
//     step kt multiplies the tiles in two slots, the loads of B(kt+1), A(kt+2) and B(kt+2) are in
//     flight, issued so that every load has at least half a step to land before it is needed.
//   * One side instruction per MFMA: a 16x16x32 MFMA keeps the matrix core busy for 16 cycles and
//     takes 4 to issue, so one load, M0 write or ds_read issued right behind it costs nothing,
//     whereas several in a row leave the matrix core idle (measured: 2720 -> 2370 cycles per
//     K-step against 2048 of pure MFMA time).
//   * LDS rows are 128 bytes (64 bf16 = eight 16-byte groups); group g of row r is stored at
//     position g ^ ((r >> 1) & 7).  LDS on gfx950 has 64 banks of 4 bytes, so two rows share a
//     bank line; this swizzle makes the 16 lanes of a ds_read_b128 phase hit 16 distinct
//     16-byte bank groups.
//   * Operand fragments are double buffered in registers (two 32-wide k-slices of 8 + 8
//     fragments); the steady-state loop is branch-free (the last two K-steps, which load nothing
//     or only B, are peeled).
//   * The MFMA is issued with the B fragment as first operand, so a lane ends up holding four
//     consecutive columns of one row of C; results are staged through LDS and written to HBM as
//     16-byte vectors, whole rows of the wavefront's block contiguous.
//   * B stored [K,N] (N a multiple of 8, N <= 2^23) runs the same kernel: the B tile lies in LDS as
//     in memory, 64 rows (k) of 256 columns, and ds_read_b64_tr_b16 transposes while reading: two
//     reads give a lane the 8 consecutive k of one column.  48 instead of 32 LDS reads per K-step,
//     still one per MFMA.
//   * K not a multiple of 64 (kernels of their own): after the loop's whole steps the last K % 64
//     columns are fetched with guarded loads, zero filled from K on, stored to LDS in the loop's
//     layout and multiplied by the same reads and MFMAs.
// General kernel (any K multiple of 8, either B layout, v_mfma_f32_32x32x16_bf16): tiles are
// fetched into registers with bounds checks and zero fill, then stored to LDS ([K,N]: 8 x 8
// blocks transposed in registers first); single buffered.  Slower; used for K < 64 and beyond
// the fast kernel's size limits.
#include <hip/hip_runtime.h>
#include <atomic>
#include <type_traits>
#include "common.h"

namespace {

constexpr int BM = 256, BN = 256, BK = 64, THREADS = 256;
constexpr int VEC_PER_THREAD = (BM * BK / 8) / THREADS;  // 16-byte vectors of one operand tile per thread = 8

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct GemmArgs {
    const uint16_t* A;
    const uint16_t* B;
    void* C;
    int64_t M, N, K;
    int32_t tiles_m, tiles_n;
};

__device__ __forceinline__ uint32_t bf16_round_bits(float f) {
    const uint32_t u = __float_as_uint(f);
    const uint32_t upper = u >> 16, lower = u & 0xffffu;
    const uint32_t r = upper + ((lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) ? 1u : 0u);
    return ((u & 0x7fffffffu) > 0x7f800000u) ? (upper | 0x0040u) : r;
}

// index (in 16-byte units) of group `cg` of row `row` in a swizzled [rows][8] tile
__device__ __forceinline__ int swz(int row, int cg) { return row * 8 + (cg ^ (row & 7)); }

// Workgroup id -> (tile_m, tile_n).  Hardware deals consecutive ids round-robin to the 8 XCDs;
// id = x + 8*q is given the q-th tile of the x-th eighth of the tile list, and the list itself
// runs down columns of 8 tile-rows so that neighbours share B panels and reuse A panels.
__device__ __forceinline__ void tile_of(int id, int tiles_m, int tiles_n, int* tm, int* tn) {
    const int total = tiles_m * tiles_n;
    int lin = id;
    if ((total & 7) == 0) lin = (id & 7) * (total >> 3) + (id >> 3);
    constexpr int GROUP = 8;
    const int per_group = GROUP * tiles_n;
    const int grp = lin / per_group;
    const int first_m = grp * GROUP;
    const int rows = tiles_m - first_m < GROUP ? tiles_m - first_m : GROUP;
    const int in = lin - grp * per_group;
    *tm = first_m + in % rows;
    *tn = in / rows;
}

template <bool B_NK, bool OUT_BF16>
__global__ void __launch_bounds__(THREADS) gemm_bf16_general_kernel(const GemmArgs p) {
    __shared__ u32x4 sA[BM * 8];
    __shared__ u32x4 sB[BN * 8];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    int tm, tn;
    tile_of(blockIdx.x, p.tiles_m, p.tiles_n, &tm, &tn);
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
    const int64_t M = p.M, N = p.N, K = p.K;

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    u32x4 ra[VEC_PER_THREAD], rb[VEC_PER_THREAD];
    const u32x4 zero = {0u, 0u, 0u, 0u};

    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int i = 0; i < VEC_PER_THREAD; ++i) {
            const int id = tid + THREADS * i;
            const int row = id >> 3, cg = id & 7;
            const int64_t gm = m0 + row, gk = k0 + cg * 8;
            ra[i] = (gm < M && gk < K) ? *reinterpret_cast<const u32x4*>(p.A + gm * K + gk) : zero;
        }
        if (B_NK) {
#pragma unroll
            for (int i = 0; i < VEC_PER_THREAD; ++i) {
                const int id = tid + THREADS * i;
                const int row = id >> 3, cg = id & 7;
                const int64_t gn = n0 + row, gk = k0 + cg * 8;
                rb[i] = (gn < N && gk < K) ? *reinterpret_cast<const u32x4*>(p.B + gn * K + gk) : zero;
            }
        } else {
#pragma unroll
            for (int i = 0; i < VEC_PER_THREAD; ++i) {   // B[K,N]: a thread holds an 8 (k) x 8 (n) block
                const int64_t gk = k0 + (tid & 7) * 8 + i, gn = n0 + (tid >> 3) * 8;
                rb[i] = (gk < K && gn < N) ? *reinterpret_cast<const u32x4*>(p.B + gk * N + gn) : zero;
            }
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int i = 0; i < VEC_PER_THREAD; ++i) {
            const int id = tid + THREADS * i;
            sA[swz(id >> 3, id & 7)] = ra[i];
        }
        if (B_NK) {
#pragma unroll
            for (int i = 0; i < VEC_PER_THREAD; ++i) {
                const int id = tid + THREADS * i;
                sB[swz(id >> 3, id & 7)] = rb[i];
            }
        } else {
            // Transpose the 8 x 8 block in registers: column e of the block becomes one 16-byte group
            // (8 consecutive k of row n) of the [n][k] tile.  v_perm_b32 picks the low or the high halves
            // of two rows' words.  The 8 lanes tid & 7 of a row n write its 8 different groups.
            const int kb = tid & 7, nv = tid >> 3;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                u32x4 col;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    col[j] = __builtin_amdgcn_perm(rb[2 * j + 1][e >> 1], rb[2 * j][e >> 1],
                                                   (e & 1) ? 0x07060302u : 0x05040100u);
                sB[swz(nv * 8 + e, kb)] = col;
            }
        }
    };

    const int64_t ksteps = (K + BK - 1) / BK;
    fetch(0);
    stage();
    __syncthreads();
    for (int64_t kt = 0; kt < ksteps; ++kt) {
        if (kt + 1 < ksteps) fetch((kt + 1) * BK);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int cg = kk * 2 + (lane >> 5);
            bf16x8 a[4], b[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                a[t] = __builtin_bit_cast(bf16x8, sA[swz(wm * 128 + t * 32 + (lane & 31), cg)]);
                b[t] = __builtin_bit_cast(bf16x8, sB[swz(wn * 128 + t * 32 + (lane & 31), cg)]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
        if (kt + 1 < ksteps) {
            stage();
            __syncthreads();
        }
    }

    // accumulator element v of a 32x32 tile: row 8*(v/4) + 4*(lane/32) + v%4, column lane%32
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t col = n0 + wn * 128 + j * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = m0 + wm * 128 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (row < M && col < N) {
                    if (OUT_BF16) reinterpret_cast<uint16_t*>(p.C)[row * N + col] = (uint16_t)bf16_round_bits(acc[i][j][v]);
                    else reinterpret_cast<float*>(p.C)[row * N + col] = acc[i][j][v];
                }
            }
        }
}


// ------------------------------------------------------------------------- fast kernel
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
constexpr int LDS_SLOTS = 5;                             // ring of operand tiles: A0 B0 A1 B1 A2 ...
constexpr int SLOT_BYTES = BM * BK * 2;                  // 32 KiB: one operand tile
constexpr int FAST_LDS_BYTES = LDS_SLOTS * SLOT_BYTES;   // 160 KiB: all of a compute unit's LDS
constexpr int64_t FAST_MAX_K = int64_t(1) << 22;         // 256 rows x K x 2 bytes must fit a 32-bit lane offset
constexpr int64_t FAST_MAX_N_KN = int64_t(1) << 23;      // B stored [K,N]: so must 128 rows x N x 2 bytes

__device__ __forceinline__ int swz64(int row, int cg) { return row * 8 + (cg ^ ((row >> 1) & 7)); }

// B stored [K,N]: 16-byte group c of row k of a tile sits at position c ^ kn_swz(k).  A transposing read
// touches rows 8q + 4h + r (q, r = 0..3) for one h, 32 bytes in each: the swizzle sends those 16 rows to 16
// different 32-byte windows.
__device__ __forceinline__ int kn_swz(int k) { return (((k >> 3) & 3) << 3) | ((k & 3) << 1); }

// One 16x16x32 MFMA, accumulator pinned to the AGPR file.  Written as inline asm: with the builtin the
// register allocator rotates the 64 accumulator quads through copies on every loop iteration.
#define LAGOM_MFMA_16x16x32(ACC, SRC_A, SRC_B) \
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(ACC) : "v"(SRC_A), "v"(SRC_B))

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) char* lds_bytes;

// B_KN = false: B stored [N,K]; true: B stored [K,N], its tiles kept in LDS as 64 rows (k) of 256 columns
// and transposed by the LDS reads.
// K_TAIL: K is not a multiple of 64; the last K % 64 columns are multiplied in a step of their own after the loop.
template <bool B_KN, bool OUT_BF16, bool K_TAIL>
__device__ __forceinline__ void fast_gemm_body(const GemmArgs& p) {
    extern __shared__ u32x4 smem[];   // LDS_SLOTS operand tiles of 2048 16-byte slots
    // Wavefronts of a communication kernel may share this wavefront's SIMD (this kernel leaves them
    // registers): let the instruction arbiter prefer the GEMM.
    __builtin_amdgcn_s_setprio(3);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    int tm, tn;
    tile_of(blockIdx.x, p.tiles_m, p.tiles_n, &tm, &tn);
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
    const int64_t M = p.M, N = p.N, K = p.K;
    const char* smem_bytes = reinterpret_cast<const char*>(smem);

    f32x4 acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.0f;

    // Load instruction d (0..7) of an operand tile fills its 16-byte slots [(d*4+wave)*64, +64):
    // lane -> row (d*4+wave)*8 + lane/8, stored group lane%8, i.e. source group (lane%8) ^ ((row>>1)&7).
    // (row>>1)&7 does not depend on d because rows of successive d differ by 32.
    // Addresses are a wave-uniform 64-bit base (first row of the tile, advanced along K) plus a 32-bit
    // byte offset per lane; rows past the edge re-read the last row.
    const int srow = wave * 8 + (lane >> 3);
    const int scg = (lane & 7) ^ ((srow >> 1) & 7);
    const char* base_a = reinterpret_cast<const char*>(p.A + m0 * K);
    // B stored [K,N]: a tile is 64 rows (k) of 512 bytes (256 n = 32 groups).  Load d fills rows
    // 8*d + 2*wave + lane/32, stored group lane%32 holding source group (lane%32) ^ kn_swz(row);
    // groups past the last column re-read the last one.  Successive K-steps are 64 rows of B apart.
    const char* base_b = reinterpret_cast<const char*>(B_KN ? p.B + n0 : p.B + n0 * K);
    const int64_t b_step = B_KN ? 2 * BK * N : 2 * BK;   // bytes from one K-step's tile of B to the next
    uint32_t a_off[8], b_off[8];
#pragma unroll
    for (int d = 0; d < 8; ++d) {
        const int64_t r = srow + 32 * d, last_a = M - 1 - m0, last_b = N - 1 - n0;
        a_off[d] = (uint32_t)(((r < last_a ? r : last_a) * K + scg * 8) * 2);
        if (B_KN) {
            const int krow = 8 * d + 2 * wave + (lane >> 5);
            const int64_t grp = (lane & 31) ^ kn_swz(krow), last_grp = (N - n0) / 8 - 1;
            b_off[d] = (uint32_t)((krow * N + (grp < last_grp ? grp : last_grp) * 8) * 2);
        } else {
            b_off[d] = (uint32_t)(((r < last_b ? r : last_b) * K + scg * 8) * 2);
        }
    }
    // LDS byte address of this wavefront's 1 KiB window of load 0 in slot 0
    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) char*)smem + wave * 1024;
    // 16 bytes per lane from global memory straight into LDS: M0 holds the LDS address of lane 0.
    auto load_now = [&](const char* sbase, uint32_t voff, int slot, int d) {
        const uint32_t la = lds0 + slot * SLOT_BYTES + d * 4096;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(la), "v"(voff), "s"(sbase) : "memory");
    };
    // main-loop form in two halves, one MFMA apart (which also is the wait state M0 needs before the load)
    auto set_m0 = [&](uint32_t slot_base, int d) { asm volatile("s_add_i32 m0, %0, %1" ::"s"(slot_base), "n"(d * 4096) : "memory"); };
    // (no immediate offset: the hardware would add it to the LDS address as well)
    auto load_m0 = [&](const char* sbase, uint32_t voff) { asm volatile("global_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase) : "memory"); };

    const int64_t ksteps = K / BK;
    // prologue: A0 -> slot 0, B0 -> slot 1, A1 -> slot 2, first half of B1 -> slot 3
#pragma unroll
    for (int d = 0; d < 8; ++d) load_now(base_a, a_off[d], 0, d);
#pragma unroll
    for (int d = 0; d < 8; ++d) load_now(base_b, b_off[d], 1, d);
    if (ksteps > 1) {
#pragma unroll
        for (int d = 0; d < 8; ++d) load_now(base_a + BK * 2, a_off[d], 2, d);
#pragma unroll
        for (int d = 0; d < 4; ++d) load_now(base_b + b_step, b_off[d], 3, d);
        asm volatile("s_waitcnt vmcnt(12)" ::: "memory");   // loads complete in issue order: A0 and B0 are in
    } else {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __builtin_amdgcn_s_barrier();

    // Fragment r of a 32-wide k-slice: lane -> row 16*r + lane%16, 16-byte group 4*slice + lane/16.
    const int arow = wm * 128 + (lane & 15), brow = wn * 128 + (lane & 15), kq = lane >> 4;
    bf16x8 fa[2][8], fb[2][8];
    // B stored [K,N]: fragment j of a k-slice is two transposing reads (h = 0, 1).  In each, lane
    // 16*q + i hands in the address of B[8q + 4h + i/4][16j + 4*(i%4) .. +3] and receives
    // B[8q + 4h + 0..3][16j + i]: together the 8 consecutive k of column 16j + lane%16 that the MFMA
    // pairs with A[row][8q .. 8q+7].  kn_frag[j]: the lane's byte offset for fragment j in a tile's slot;
    // slice and h move it by whole rows (16 KiB, 2 KiB), which the swizzle does not see.
    s16x4 fbh[B_KN ? 2 : 1][B_KN ? 8 : 1][2];
    uint32_t kn_frag[B_KN ? 8 : 1];
    if (B_KN) {
        const int i = lane & 15, r = i >> 2;
        const int krow = 8 * kq + r;                                   // slice 0, h = 0
        const int grp0 = wn * 16 + ((i & 3) >> 1);                     // source group of fragment 0
#pragma unroll
        for (int j = 0; j < 8; ++j)
            kn_frag[j] = (uint32_t)(krow * 512 + (((grp0 + 2 * j) ^ kn_swz(krow)) << 4) + 8 * (i & 1));
    }
    // r: 0..7 = A0..A7, 8..15 = B0..B7; half: which of the two reads of a [K,N] B fragment
    auto read_frag = [&](const u32x4* sa, const u32x4* sb, int ks, int r, int buf, int half) {
        if (r < 8) {
            fa[buf][r] = __builtin_bit_cast(bf16x8, sa[swz64(arow + r * 16, ks * 4 + kq)]);
        } else if (!B_KN) {
            fb[buf][r - 8] = __builtin_bit_cast(bf16x8, sb[swz64(brow + (r - 8) * 16, ks * 4 + kq)]);
        } else {
            typedef s16x4 __attribute__((address_space(3))) * tr_ptr;
            fbh[buf][r - 8][half] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (tr_ptr)((lds_bytes)(const char*)sb + kn_frag[r - 8] + ks * 16384 + half * 2048));
        }
    };
    auto b_frag = [&](int buf, int j) -> bf16x8 {
        if (!B_KN) return fb[buf][j];
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(fbh[buf][j][0], fbh[buf][j][1], 0, 1, 2, 3, 4, 5, 6, 7));
    };
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        read_frag(smem, smem + SLOT_BYTES / 16, 0, r, 0, 0);
        if (B_KN && r >= 8) read_frag(smem, smem + SLOT_BYTES / 16, 0, r, 0, 1);
    }

    // One K-step = 2 k-slices x 8 groups x 8 MFMAs (group g: A fragment g against the 8 B fragments).
    // MORE1 / MORE2: tiles kt+1 / kt+2 exist (compile-time, so that the steady-state loop has no
    // branches; the last two K-steps are peeled).  Every MFMA is followed by at most one other
    // instruction, which issues while the matrix core works on that MFMA:
    //   loads   one per group, M0 after the group's first MFMA and the load after its third:
    //           groups 0-3 second half of B(kt+1); 4-11 A(kt+2) into the fifth slot; 12-15 first half
    //           of B(kt+2) into the slot A(kt) has just left.
    //   reads   slice 0: two fragments of slice 1 per group; slice 1, groups 4-7: four fragments per
    //           group of slice 0 of tile kt+1, in the order the next step consumes them.
    //   barrier in front of group 12: by then this wavefront holds every fragment of tile kt in
    //           registers and tile kt+1 has landed (the 8 youngest loads, A(kt+2), may still fly), so
    //           after the barrier tile kt's slots are free and tile kt+1 may be read.
    constexpr int kReadOrder[16] = {0, 8, 9, 10, 11, 12, 13, 14, 15, 1, 2, 3, 4, 5, 6, 7};   // A0, B0..B7, A1..A7
    // Byte offsets of the slots of A(kt), B(kt), A(kt+1), B(kt+1), A(kt+2).  Advancing by one K-step moves
    // every role two slots along a ring of five, which is a pure rotation of these five values.
    uint32_t o_a = 0, o_b = SLOT_BYTES, o_a1 = 2 * SLOT_BYTES, o_b1 = 3 * SLOT_BYTES, o_a2 = 4 * SLOT_BYTES;
    const char* g_a = base_a + 2 * (BK * 2);   // &A[m0][(kt+2)*64]
    const char* g_b = base_b + b_step;         // tile kt+1 of B; tile kt+2 is reached through b_off_next
    uint32_t b_off_next[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) b_off_next[d] = b_off[d] + (uint32_t)b_step;
    // Fragment reads of one k-slice in the order the MFMAs consume them.  [N,K]: 16 reads, A0, B0..B7,
    // A1..A7.  [K,N]: 24 reads, every B fragment being two.
    constexpr int kReads = B_KN ? 24 : 16;
    auto read_nth = [&](const u32x4* sa, const u32x4* sb, int ks, int n, int buf) {
        if (!B_KN) read_frag(sa, sb, ks, kReadOrder[n], buf, 0);
        else if (n == 0) read_frag(sa, sb, ks, 0, buf, 0);
        else if (n <= 16) read_frag(sa, sb, ks, 8 + (n - 1) / 2, buf, (n - 1) & 1);
        else read_frag(sa, sb, ks, n - 16, buf, 0);
    };
    auto step = [&](auto more1_c, auto more2_c) {
        constexpr bool more1 = decltype(more1_c)::value, more2 = decltype(more2_c)::value;
        const u32x4* sa = reinterpret_cast<const u32x4*>(smem_bytes + o_a);
        const u32x4* sb = reinterpret_cast<const u32x4*>(smem_bytes + o_b);
        const u32x4* sa1 = reinterpret_cast<const u32x4*>(smem_bytes + o_a1);
        const u32x4* sb1 = reinterpret_cast<const u32x4*>(smem_bytes + o_b1);
        const uint32_t l_b1 = lds0 + o_b1, l_a2 = lds0 + o_a2, l_a = lds0 + o_a;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
            for (int g = 0; g < 8; ++g) {
                const int q = ks * 8 + g;
                if (q == 12) {
                    if (more2) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
                    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    __builtin_amdgcn_s_barrier();
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    // B fragment first: the lane's 4 results are C[row lane%16][4 consecutive columns]
                    LAGOM_MFMA_16x16x32(acc[g][j], b_frag(ks, j), fa[ks][g]);
                    __builtin_amdgcn_sched_barrier(0);
                    if (j == 0) {
                        if (q < 4) { if (more1) set_m0(l_b1, 4 + q); }
                        else if (q < 12) { if (more2) set_m0(l_a2, q - 4); }
                        else { if (more2) set_m0(l_a, q - 12); }
                    }
                    if (j == 2) {
                        if (q < 4) { if (more1) load_m0(g_b, b_off[4 + q]); }
                        else if (q < 12) { if (more2) load_m0(g_a, a_off[q - 4]); }
                        else { if (more2) load_m0(g_b, b_off_next[q - 12]); }
                    }
                    if (ks == 0) {   // slice 1 of this tile: 2 (3) reads per group
                        if (j == 3) read_nth(sa, sb, 1, (kReads / 8) * g, 1);
                        if (j == 5) read_nth(sa, sb, 1, (kReads / 8) * g + 1, 1);
                        if (B_KN && j == 6) read_nth(sa, sb, 1, 3 * g + 2, 1);
                    } else if (more1 && g >= 4) {   // slice 0 of tile kt+1: 4 (6) reads per group
                        if (!B_KN) {
                            if (j & 1) read_nth(sa1, sb1, 0, (g - 4) * 4 + (j >> 1), 0);
                        } else {
                            constexpr int kSlot[8] = {-1, 0, -1, 1, 2, 3, 4, 5};
                            if (kSlot[j] >= 0) read_nth(sa1, sb1, 0, (g - 4) * 6 + kSlot[j], 0);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        const uint32_t t_a = o_a, t_b = o_b;
        o_a = o_a1; o_b = o_b1; o_a1 = o_a2; o_b1 = t_a; o_a2 = t_b;
        g_a += BK * 2;
        g_b += b_step;
    };
    int kt = 0;
    const int nk = (int)ksteps;
    for (; kt + 2 < nk; ++kt) step(std::true_type{}, std::true_type{});
    if (kt + 1 < nk) { step(std::true_type{}, std::false_type{}); ++kt; }
    if (kt < nk) step(std::false_type{}, std::false_type{});
    if (K_TAIL) {
        // The last K % 64 columns: fetched with ordinary guarded loads (zeros from K on, in both operands),
        // put into the first two slots in the layout the loop uses, and multiplied by the same fragment
        // reads and MFMAs.  Every wavefront is past the last step's barrier, behind which nothing reads
        // LDS and no LDS-direct load is in flight.
        const int64_t kbase = ksteps * BK;
        u32x4 ta[8], tb[8];
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int id = tid + THREADS * i;
            const int64_t gm = m0 + (id >> 3), gk = kbase + (id & 7) * 8;
            ta[i] = (gm < M && gk < K) ? *reinterpret_cast<const u32x4*>(p.A + gm * K + gk) : zero;
            if (B_KN) {
                const int64_t bk = kbase + (id >> 5), gn = n0 + (id & 31) * 8;
                tb[i] = (bk < K && gn < N) ? *reinterpret_cast<const u32x4*>(p.B + bk * N + gn) : zero;
            } else {
                const int64_t gn = n0 + (id >> 3);
                tb[i] = (gn < N && gk < K) ? *reinterpret_cast<const u32x4*>(p.B + gn * K + gk) : zero;
            }
        }
        u32x4* slot_a = smem;
        u32x4* slot_b = smem + SLOT_BYTES / 16;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int id = tid + THREADS * i;
            slot_a[swz64(id >> 3, id & 7)] = ta[i];
            if (B_KN) slot_b[(id >> 5) * 32 + ((id & 31) ^ kn_swz(id >> 5))] = tb[i];
            else slot_b[swz64(id >> 3, id & 7)] = tb[i];
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            if (ks == 1 && K - kbase <= 32) break;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                read_frag(slot_a, slot_b, ks, r, 0, 0);
                if (B_KN && r >= 8) read_frag(slot_a, slot_b, ks, r, 0, 1);
            }
#pragma unroll
            for (int g = 0; g < 8; ++g)
#pragma unroll
                for (int j = 0; j < 8; ++j) LAGOM_MFMA_16x16x32(acc[g][j], b_frag(0, j), fa[0][g]);
        }
    }
    // The compiler does not see an MFMA inside the asm statements and therefore adds none of the wait
    // states an accumulator read needs after one: give the last results their cycles here, and make
    // every later use of an accumulator depend on a statement that follows these cycles.
    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) asm volatile("" : "+a"(acc[i][j]));
    __builtin_amdgcn_s_barrier();   // every wavefront is past its last LDS read before the slots are reused below

    // Epilogue.  acc[i][j][v] is row 16*i + lane%16, column 16*j + 4*(lane/16) + v of the wavefront's
    // 128 x 128 block.  The block is staged in the wavefront's own 32 KiB of LDS as rows of ROW_BYTES
    // (16-byte group c of row r stored at c ^ (r & 15)) and written out as 16-byte vectors, whole rows
    // of the block contiguous: all 128 rows at once for bf16, 64 rows per pass for fp32.  A wavefront
    // reads back only what it wrote itself, and LDS serves one wavefront's accesses in order, so the
    // passes need no waits between them beyond the data dependencies.
    constexpr int ESZ = OUT_BF16 ? 2 : 4;
    constexpr int PASSES = OUT_BF16 ? 1 : 2;
    constexpr int ROW_BYTES = 128 * ESZ, GROUPS = ROW_BYTES / 16, ROWS_PER_READ = 64 / GROUPS, VEC = 16 / ESZ;
    const int r_in = lane & 15, c_q = 4 * (lane >> 4);
    char* st = reinterpret_cast<char*>(smem) + wave * SLOT_BYTES;
    const bool interior = m0 + BM <= M && n0 + BN <= N;
    const bool vector_ok = (N % VEC) == 0;
    const int rd_row = lane / GROUPS, rd_cv = lane % GROUPS;
    const int64_t gcol = n0 + wn * 128 + rd_cv * VEC;
#pragma unroll
    for (int pass = 0; pass < PASSES; ++pass) {
#pragma unroll
        for (int ii = 0; ii < 8 / PASSES; ++ii)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int i = pass * (8 / PASSES) + ii;
                const int r = ii * 16 + r_in;
                const int cb = (j * 16 + c_q) * ESZ;          // byte offset of the first of four consecutive columns
                char* dst = st + r * ROW_BYTES + (((cb >> 4) ^ (r & 15)) << 4) + (cb & 15);
                if (OUT_BF16) {
                    const bf16x2 lo = __builtin_convertvector(f32x2{acc[i][j][0], acc[i][j][1]}, bf16x2);
                    const bf16x2 hi = __builtin_convertvector(f32x2{acc[i][j][2], acc[i][j][3]}, bf16x2);
                    uint2 v;
                    v.x = __builtin_bit_cast(uint32_t, lo);
                    v.y = __builtin_bit_cast(uint32_t, hi);
                    *reinterpret_cast<uint2*>(dst) = v;
                } else {
                    *reinterpret_cast<f32x4*>(dst) = acc[i][j];
                }
            }
        const int64_t row0 = m0 + wm * 128 + pass * (128 / PASSES) + rd_row;
#pragma unroll
        for (int tb = 0; tb < 4; ++tb) {   // eight reads in flight, then eight stores
            u32x4 val[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int r = rd_row + ROWS_PER_READ * (tb * 8 + e);
                val[e] = *reinterpret_cast<const u32x4*>(st + r * ROW_BYTES + ((rd_cv ^ (r & 15)) << 4));
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int64_t grow = row0 + ROWS_PER_READ * (tb * 8 + e);
                char* out = reinterpret_cast<char*>(p.C) + (grow * N + gcol) * ESZ;
                if (vector_ok) {
                    if (interior || (grow < M && gcol < N)) __builtin_nontemporal_store(val[e], reinterpret_cast<u32x4*>(out));
                } else if (grow < M) {
#pragma unroll
                    for (int k = 0; k < VEC; ++k)
                        if (gcol + k < N) {
                            if (OUT_BF16) reinterpret_cast<uint16_t*>(out)[k] = (uint16_t)(val[e][k >> 1] >> (16 * (k & 1)));
                            else reinterpret_cast<uint32_t*>(out)[k] = val[e][k];
                        }
                }
            }
        }
    }
}

template <bool OUT_BF16>
__global__ void __launch_bounds__(THREADS) gemm_bf16_nk_kernel(const GemmArgs p) { fast_gemm_body<false, OUT_BF16, false>(p); }
template <bool OUT_BF16>
__global__ void __launch_bounds__(THREADS) gemm_bf16_kn_kernel(const GemmArgs p) { fast_gemm_body<true, OUT_BF16, false>(p); }
// K >= 64 and not a multiple of 64 (kernels of their own: the extra step costs registers the others leave free)
template <bool OUT_BF16>
__global__ void __launch_bounds__(THREADS) gemm_bf16_nk_tail_kernel(const GemmArgs p) { fast_gemm_body<false, OUT_BF16, true>(p); }
template <bool OUT_BF16>
__global__ void __launch_bounds__(THREADS) gemm_bf16_kn_tail_kernel(const GemmArgs p) { fast_gemm_body<true, OUT_BF16, true>(p); }

// ------------------------------------------------------------------------- small-tile kernels
// 128 x 128 x 64 and 256 x 128 x 64 tiles for products with too few 256 x 256 tiles to fill the chip.
// Same workgroup (4 wavefronts, 2 x 2; a wavefront owns NI x 4 MFMA tiles, NI = 4 or 8, i.e. 64 or 128
// accumulators), same LDS-direct loads, row layout and swizzles as the large kernel.  LDS holds a ring of
// A+B tile pairs: five for NI = 4 (a K-step is only 32 MFMAs long, loads run four to five steps ahead),
// three for NI = 8.  One barrier per K-step, in its middle.
constexpr int SBN = 128;
constexpr int S_B_BYTES = SBN * BK * 2;                   // 16 KiB
template <int NI> struct SmallTile {
    static constexpr int BM_ = 32 * NI;                   // rows of a tile
    static constexpr int A_BYTES = BM_ * BK * 2;          // 16 or 32 KiB
    static constexpr int STAGE_BYTES = A_BYTES + S_B_BYTES;
    static constexpr int STAGES = NI == 4 ? 5 : 3;
    static constexpr int AHEAD = STAGES - 1;
    static constexpr int LA = NI, LB = 4;                 // load instructions per wavefront for an A / a B tile
    static_assert(STAGES * STAGE_BYTES <= FAST_LDS_BYTES, "the ring fits the LDS");
};
constexpr int SBM = SmallTile<4>::BM_, MBM = SmallTile<8>::BM_;

// B stored [K,N]: a B tile is 64 rows (k) of 256 bytes (128 n = 16 groups); group c of row k sits at
// c ^ kn_swz128(k), which spreads the rows of a transposing read over the 8 32-byte windows of a row.
__device__ __forceinline__ int kn_swz128(int k) { return (((k >> 3) & 1) << 3) | ((k & 3) << 1); }

// K_TAIL: K is not a multiple of 64; the last K % 64 columns get a step of their own (see the large kernel).
template <int NI, bool B_KN, bool OUT_BF16, bool K_TAIL>
__device__ __forceinline__ void small_gemm_body(const GemmArgs& p) {
    typedef SmallTile<NI> T;
    constexpr int S_STAGES = T::STAGES, S_AHEAD = T::AHEAD, S_STAGE_BYTES = T::STAGE_BYTES, S_OPERAND_BYTES = T::A_BYTES;
    constexpr int LA = T::LA, LB = T::LB, PER_TILE = LA + LB;
    extern __shared__ u32x4 smem[];
    __builtin_amdgcn_s_setprio(3);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    int tm, tn;
    tile_of(blockIdx.x, p.tiles_m, p.tiles_n, &tm, &tn);
    const int64_t m0 = (int64_t)tm * T::BM_, n0 = (int64_t)tn * SBN;
    const int64_t M = p.M, N = p.N, K = p.K;
    const char* smem_bytes = reinterpret_cast<const char*>(smem);

    f32x4 acc[NI][4];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // load d of an operand tile: rows (d*4 + wave)*8 + lane/8, as in the large kernel
    const int srow = wave * 8 + (lane >> 3);
    const int scg = (lane & 7) ^ ((srow >> 1) & 7);
    const char* g_a = reinterpret_cast<const char*>(p.A + m0 * K);
    const char* g_b = reinterpret_cast<const char*>(B_KN ? p.B + n0 : p.B + n0 * K);
    const int64_t b_step = B_KN ? 2 * BK * N : 2 * BK;
    uint32_t a_off[LA], b_off[LB];
#pragma unroll
    for (int d = 0; d < LA; ++d) {
        const int64_t r = srow + 32 * d, last_a = M - 1 - m0;
        a_off[d] = (uint32_t)(((r < last_a ? r : last_a) * K + scg * 8) * 2);
    }
#pragma unroll
    for (int d = 0; d < LB; ++d) {
        const int64_t r = srow + 32 * d, last_b = N - 1 - n0;
        if (B_KN) {   // load d fills rows 16*d + 4*wave + lane/16 of the [64][128] tile, stored group lane%16
            const int krow = 16 * d + 4 * wave + (lane >> 4);
            const int64_t grp = (lane & 15) ^ kn_swz128(krow), last_grp = (N - n0) / 8 - 1;
            b_off[d] = (uint32_t)((krow * N + (grp < last_grp ? grp : last_grp) * 8) * 2);
        } else {
            b_off[d] = (uint32_t)(((r < last_b ? r : last_b) * K + scg * 8) * 2);
        }
    }
    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) char*)smem + wave * 1024;
    auto load_tile = [&](int stage) {   // the tile g_a / g_b point at, then advance them one K-step
        const uint32_t base = lds0 + stage * S_STAGE_BYTES;
#pragma unroll
        for (int d = 0; d < LA; ++d)
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(base + d * 4096), "v"(a_off[d]), "s"(g_a) : "memory");
#pragma unroll
        for (int d = 0; d < LB; ++d)
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(base + S_OPERAND_BYTES + d * 4096), "v"(b_off[d]), "s"(g_b) : "memory");
        g_a += BK * 2;
        g_b += b_step;
    };

    const int nk = (int)(K / BK);
    for (int t = 0; t < S_AHEAD && t < nk; ++t) load_tile(t);
    // Tile t >= AHEAD is loaded in two halves: A behind the barrier of step t-STAGES, B in the first half of
    // step t-AHEAD (g_a / g_b point at the next tile to load of their operand).
    auto set_m0 = [&](uint32_t lds) { asm volatile("s_mov_b32 m0, %0" ::"s"(lds) : "memory"); };
    auto load_m0 = [&](const char* sbase, uint32_t voff) { asm volatile("global_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase) : "memory"); };
    if (S_AHEAD < nk) {
#pragma unroll
        for (int d = 0; d < LA; ++d)
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds0 + S_AHEAD * S_STAGE_BYTES + d * 4096), "v"(a_off[d]), "s"(g_a) : "memory");
        g_a += BK * 2;
    }

    const int arow = wm * (16 * NI) + (lane & 15), brow = wn * 64 + (lane & 15), kq = lane >> 4;
    bf16x8 fa[2][NI];
    bf16x8 fb[2][4];             // fragments of the two 32-wide k-slices, read half a K-step before their MFMAs
    s16x4 fbh[B_KN ? 2 : 1][B_KN ? 4 : 1][2];
    // B stored [K,N]: fragment j is two transposing reads (rows 8q + 4h + i/4 of the slice, h = 0, 1; see the
    // large kernel); kn_frag[j] is the lane's byte offset for h = 0 in slice 0
    uint32_t kn_frag[B_KN ? 4 : 1];
    if (B_KN) {
        const int i = lane & 15, krow = 8 * kq + (i >> 2);
        const int grp0 = wn * 8 + ((i & 3) >> 1);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            kn_frag[j] = (uint32_t)(krow * 256 + (((grp0 + 2 * j) ^ kn_swz128(krow)) << 4) + 8 * (i & 1));
    }
    constexpr int UNITS = NI + 4;
    // read unit u of a slice, in the order the MFMAs consume them: A0, B0, B1, B2, B3, A1, A2, ...
    auto read_unit = [&](uint32_t stage_bytes, int ks, int u) {
        const u32x4* sa = reinterpret_cast<const u32x4*>(smem_bytes + stage_bytes);
        const u32x4* sb = sa + S_OPERAND_BYTES / 16;
        if (u == 0 || u >= 5) {
            const int r = u == 0 ? 0 : u - 4;
            fa[ks][r] = __builtin_bit_cast(bf16x8, sa[swz64(arow + r * 16, ks * 4 + kq)]);
        } else if (!B_KN) {
            fb[ks][u - 1] = __builtin_bit_cast(bf16x8, sb[swz64(brow + (u - 1) * 16, ks * 4 + kq)]);
        } else {
            typedef s16x4 __attribute__((address_space(3))) * tr_ptr;
            const lds_bytes at = (lds_bytes)(const char*)sb + kn_frag[u - 1] + ks * 8192;
            fbh[ks][u - 1][0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_ptr)at);
            fbh[ks][u - 1][1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_ptr)(at + 1024));
        }
    };
    auto b_frag = [&](int ks, int j) -> bf16x8 {
        if (!B_KN) return fb[ks][j];
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(fbh[ks][j][0], fbh[ks][j][1], 0, 1, 2, 3, 4, 5, 6, 7));
    };
    // loads complete in issue order: wait until all but the youngest `tiles` whole tiles have landed
    auto wait_all_but = [&](int tiles) {
        if (tiles >= 3 && S_AHEAD > 3) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(3 * PER_TILE) : "memory");
        else if (tiles >= 2 && S_AHEAD > 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * PER_TILE) : "memory");
        else if (tiles >= 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PER_TILE) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    };
    wait_all_but(nk - 1 < S_AHEAD - 1 ? nk - 1 : S_AHEAD - 1);   // tile 0 (the A half of tile AHEAD, if any, may fly on as well)
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int u = 0; u < UNITS; ++u) read_unit(0, 0, u);

    // One K-step = 2 k-slices x 4*NI MFMAs, each MFMA followed by at most one side instruction (a B fragment
    // of the [K,N] layout being two reads):
    //   first half   NI + 4 fragment reads of slice 1; then the B half of tile kt+AHEAD (M0 write and load
    //                alternating)
    //   barrier      behind vmcnt: tile kt+1 has landed for every wavefront; nobody reads tile kt any more
    //                (its fragments are in registers), so its slot can take the A half of tile kt+STAGES
    //   second half  NI + 4 fragment reads of slice 0 of tile kt+1; then the A half of tile kt+STAGES
    // LOAD_B / LOAD_A / NEXT: tiles kt+AHEAD / kt+STAGES / kt+1 exist (compile time: no branch inside a step).
    uint32_t o_cur = 0, o_next = S_STAGE_BYTES, o_b4 = S_AHEAD * S_STAGE_BYTES;   // byte offsets of the slots of tiles kt, kt+1, kt+4
    int kt = 0;
    auto step = [&](auto load_b_c, auto load_a_c, auto next_c) {
        constexpr bool LOAD_B = decltype(load_b_c)::value, LOAD_A = decltype(load_a_c)::value, NEXT = decltype(next_c)::value;
        const uint32_t l_b = lds0 + o_b4 + S_OPERAND_BYTES, l_a = lds0 + o_cur;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            if (ks == 1) {
                // issued and not needed yet: the whole tiles kt+2 .. kt+AHEAD that exist
                if (LOAD_B) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S_AHEAD - 1) * PER_TILE) : "memory");
                else if (NEXT) wait_all_but(nk - 2 - kt);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int sl = i * 4 + j;     // slot within the half
                    // B fragment first: a lane holds 4 consecutive columns of one row
                    LAGOM_MFMA_16x16x32(acc[i][j], b_frag(ks, j), fa[ks][i]);
                    __builtin_amdgcn_sched_barrier(0);
                    if (sl < UNITS) {
                        if (ks == 0) read_unit(o_cur, 1, sl);
                        else if (NEXT) read_unit(o_next, 0, sl);
                    } else {
                        const int d = (sl - UNITS) >> 1, odd = (sl - UNITS) & 1;
                        if (ks == 0 && LOAD_B && d < LB) { if (odd) load_m0(g_b, b_off[d]); else set_m0(l_b + d * 4096); }
                        if (ks == 1 && LOAD_A && d < LA) { if (odd) load_m0(g_a, a_off[d]); else set_m0(l_a + d * 4096); }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
        }
        if (LOAD_B) g_b += b_step;
        if (LOAD_A) g_a += BK * 2;
        o_cur = o_next;
        o_next = o_next + S_STAGE_BYTES == S_STAGES * S_STAGE_BYTES ? 0 : o_next + S_STAGE_BYTES;
        o_b4 = o_b4 + S_STAGE_BYTES == S_STAGES * S_STAGE_BYTES ? 0 : o_b4 + S_STAGE_BYTES;
        ++kt;
    };
    while (kt + S_STAGES < nk) step(std::true_type{}, std::true_type{}, std::true_type{});
    // at most STAGES steps are left, peeled in straight-line code (a loop over step variants makes the register
    // allocator copy accumulators between them, with none of the wait states a copy behind an MFMA needs)
    if (kt + S_AHEAD < nk) step(std::true_type{}, std::false_type{}, std::true_type{});
    if (kt + 1 < nk) step(std::false_type{}, std::false_type{}, std::true_type{});
    if (S_AHEAD > 2) {
        if (kt + 1 < nk) step(std::false_type{}, std::false_type{}, std::true_type{});
        if (kt + 1 < nk) step(std::false_type{}, std::false_type{}, std::true_type{});
    }
    if (kt < nk) step(std::false_type{}, std::false_type{}, std::false_type{});
    if (K_TAIL) {
        // Every wavefront is past the barrier of the last step, behind which nothing reads LDS and no
        // LDS-direct load is in flight: the first slot takes the zero-filled rest of K in the loop's layout.
        const int64_t kbase = (int64_t)nk * BK;
        u32x4 ta[LA], tb[LB];
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            const int id = tid + THREADS * i;
            const int64_t gm = m0 + (id >> 3), gk = kbase + (id & 7) * 8;
            ta[i] = (gm < M && gk < K) ? *reinterpret_cast<const u32x4*>(p.A + gm * K + gk) : zero;
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int id = tid + THREADS * i;
            if (B_KN) {
                const int64_t bk = kbase + (id >> 4), gn = n0 + (id & 15) * 8;
                tb[i] = (bk < K && gn < N) ? *reinterpret_cast<const u32x4*>(p.B + bk * N + gn) : zero;
            } else {
                const int64_t gn = n0 + (id >> 3), gk = kbase + (id & 7) * 8;
                tb[i] = (gn < N && gk < K) ? *reinterpret_cast<const u32x4*>(p.B + gn * K + gk) : zero;
            }
        }
        u32x4* slot_b = smem + S_OPERAND_BYTES / 16;
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            const int id = tid + THREADS * i;
            smem[swz64(id >> 3, id & 7)] = ta[i];
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int id = tid + THREADS * i;
            if (B_KN) slot_b[(id >> 4) * 16 + ((id & 15) ^ kn_swz128(id >> 4))] = tb[i];
            else slot_b[swz64(id >> 3, id & 7)] = tb[i];
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            if (ks == 1 && K - kbase <= 32) break;
#pragma unroll
            for (int u = 0; u < UNITS; ++u) read_unit(0, 0 + ks, u);
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) LAGOM_MFMA_16x16x32(acc[i][j], b_frag(ks, j), fa[ks][i]);
        }
    }
    // wait states behind the last inline-asm MFMA, as in the large kernel
    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) asm volatile("" : "+a"(acc[i][j]));
    __builtin_amdgcn_s_barrier();   // every wavefront is past its last LDS read before the ring is reused below

    // Epilogue: acc[i][j][v] is row 16*i + lane%16, column 16*j + 4*(lane/16) + v of the wavefront's 16*NI x 64
    // block, staged in the wavefront's own LDS as rows of ROW_BYTES (16-byte group c of row r at c ^ (r % GROUPS))
    // and written out as 16-byte vectors, whole rows of the block contiguous.
    constexpr int ESZ = OUT_BF16 ? 2 : 4;
    constexpr int ROW_BYTES = 64 * ESZ, GROUPS = ROW_BYTES / 16, ROWS_PER_READ = 64 / GROUPS, VEC = 16 / ESZ;
    constexpr int WROWS = 16 * NI;
    static_assert(4 * WROWS * ROW_BYTES <= T::STAGES * T::STAGE_BYTES, "the staging areas fit the ring");
    char* st = reinterpret_cast<char*>(smem) + wave * (WROWS * ROW_BYTES);
    const int r_in = lane & 15, c_q = 4 * (lane >> 4);
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = i * 16 + r_in;
            const int cb = (j * 16 + c_q) * ESZ;
            char* dst = st + r * ROW_BYTES + (((cb >> 4) ^ (r & (GROUPS - 1))) << 4) + (cb & 15);
            if (OUT_BF16) {
                const bf16x2 lo = __builtin_convertvector(f32x2{acc[i][j][0], acc[i][j][1]}, bf16x2);
                const bf16x2 hi = __builtin_convertvector(f32x2{acc[i][j][2], acc[i][j][3]}, bf16x2);
                uint2 v;
                v.x = __builtin_bit_cast(uint32_t, lo);
                v.y = __builtin_bit_cast(uint32_t, hi);
                *reinterpret_cast<uint2*>(dst) = v;
            } else {
                *reinterpret_cast<f32x4*>(dst) = acc[i][j];
            }
        }
    const bool interior = m0 + T::BM_ <= M && n0 + SBN <= N;
    const bool vector_ok = (N % VEC) == 0;
    const int rd_row = lane / GROUPS, rd_cv = lane % GROUPS;
    const int64_t gcol = n0 + wn * 64 + rd_cv * VEC;
    const int64_t row0 = m0 + wm * WROWS + rd_row;
#pragma unroll
    for (int e = 0; e < WROWS / ROWS_PER_READ; ++e) {   // each read covers ROWS_PER_READ whole rows of the block
        const int r = rd_row + ROWS_PER_READ * e;
        const u32x4 val = *reinterpret_cast<const u32x4*>(st + r * ROW_BYTES + ((rd_cv ^ (r & (GROUPS - 1))) << 4));
        const int64_t grow = row0 + ROWS_PER_READ * e;
        char* out = reinterpret_cast<char*>(p.C) + (grow * N + gcol) * ESZ;
        if (vector_ok) {
            if (interior || (grow < M && gcol < N)) __builtin_nontemporal_store(val, reinterpret_cast<u32x4*>(out));
        } else if (grow < M) {
#pragma unroll
            for (int k = 0; k < VEC; ++k)
                if (gcol + k < N) {
                    if (OUT_BF16) reinterpret_cast<uint16_t*>(out)[k] = (uint16_t)(val[k >> 1] >> (16 * (k & 1)));
                    else reinterpret_cast<uint32_t*>(out)[k] = val[k];
                }
        }
    }
}

template <bool OUT_BF16>
__global__ void __launch_bounds__(THREADS) gemm_bf16_nk128_kernel(const GemmArgs p) { small_gemm_body<4, false, OUT_BF16, false>(p); }
template <bool OUT_BF16>
__global__ void __launch_bounds__(THREADS) gemm_bf16_kn128_kernel(const GemmArgs p) { small_gemm_body<4, true, OUT_BF16, false>(p); }
// 256 x 128 tiles
template <bool OUT_BF16>
__global__ void __launch_bounds__(THREADS) gemm_bf16_nk256x128_kernel(const GemmArgs p) { small_gemm_body<8, false, OUT_BF16, false>(p); }
template <bool OUT_BF16>
__global__ void __launch_bounds__(THREADS) gemm_bf16_kn256x128_kernel(const GemmArgs p) { small_gemm_body<8, true, OUT_BF16, false>(p); }
// K >= 64 and not a multiple of 64
template <bool OUT_BF16>
__global__ void __launch_bounds__(THREADS) gemm_bf16_nk128_tail_kernel(const GemmArgs p) { small_gemm_body<4, false, OUT_BF16, true>(p); }
template <bool OUT_BF16>
__global__ void __launch_bounds__(THREADS) gemm_bf16_kn128_tail_kernel(const GemmArgs p) { small_gemm_body<4, true, OUT_BF16, true>(p); }
template <bool OUT_BF16>
__global__ void __launch_bounds__(THREADS) gemm_bf16_nk256x128_tail_kernel(const GemmArgs p) { small_gemm_body<8, false, OUT_BF16, true>(p); }
template <bool OUT_BF16>
__global__ void __launch_bounds__(THREADS) gemm_bf16_kn256x128_tail_kernel(const GemmArgs p) { small_gemm_body<8, true, OUT_BF16, true>(p); }

template <void (*KERNEL)(const GemmArgs)>
int launch_fast(const GemmArgs& a, dim3 grid, hipStream_t st) {
    // set once per kernel (and per device: a process may drive several); a failure is not remembered
    static std::atomic<uint64_t> done_on_device{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) dev = 63;
    const uint64_t bit = uint64_t{1} << dev;
    if (dev == 63 || !(done_on_device.load(std::memory_order_acquire) & bit)) {
        const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(KERNEL),
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, FAST_LDS_BYTES);
        if (attr != hipSuccess) return lagom::fail(LAGOM_EHIP, "gemm: cannot raise the LDS limit: %s", hipGetErrorString(attr));
        done_on_device.fetch_or(bit, std::memory_order_release);
    }
    hipLaunchKernelGGL(KERNEL, grid, dim3(THREADS), FAST_LDS_BYTES, st, a);
    return LAGOM_OK;
}

// The smallest tile that still covers C in one round of workgroups (256 compute units): 128 x 128, else
// 256 x 128, else 256 x 256.  Fewer, larger tiles would leave compute units idle; smaller tiles in several
// rounds lose more to their lower arithmetic intensity than they gain.
enum Tiling { TILE_128x128, TILE_256x128, TILE_256x256 };
Tiling choose_tiling(int64_t M, int64_t N, int64_t K) {
    if (K < BK || K > FAST_MAX_K) return TILE_256x256;
    const int64_t cols = (N + SBN - 1) / SBN;
    if (((M + SBM - 1) / SBM) * cols <= 256) return TILE_128x128;
    if (((M + MBM - 1) / MBM) * cols <= 256) return TILE_256x128;
    return TILE_256x256;
}

}  // namespace

namespace lagom {
int check_gemm_args(const void* A, const void* B, const void* C, int64_t M, int64_t N, int64_t K, int out_dt) {
    if (!A || !B || !C) return fail(LAGOM_EINVAL, "null matrix pointer");
    if (M < 1 || N < 1 || K < 1) return fail(LAGOM_EINVAL, "M, N, K must be positive");
    if (M > (1 << 24) || N > (1 << 24) || K > (1 << 24)) return fail(LAGOM_EINVAL, "dimension above 2^24");
    if (K % 8) return fail(LAGOM_EINVAL, "K=%lld must be a multiple of 8", (long long)K);
    if (elem_size(out_dt) == 0) return fail(LAGOM_EINVAL, "unknown output dtype %d", out_dt);
    if (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C) & 15) return fail(LAGOM_EALIGN, "matrix pointer not 16-byte aligned");
    return LAGOM_OK;
}
}  // namespace lagom

extern "C" int lagom_gemm_describe(int64_t M, int64_t N, int64_t K, lagom_dtype out_dt, lagom_gemm_geometry* out) {
    if (!out || M < 1 || N < 1 || K < 1 || lagom::elem_size(out_dt) == 0) return lagom::fail(LAGOM_EINVAL, "bad argument");
    // the tiling lagom_gemm uses for this shape (it does not depend on B's layout)
    const Tiling tiling = choose_tiling(M, N, K);
    const int64_t bm = tiling == TILE_128x128 ? SBM : BM, bn = tiling == TILE_256x256 ? BN : SBN;
    const int64_t tm = (M + bm - 1) / bm, tn = (N + bn - 1) / bn;
    out->mu = tm * tn;
    out->tb = 1;   // either kernel takes all of a compute unit's LDS: one workgroup per compute unit
    out->d_bytes = (double)(bm + bn) * (double)K * 2.0 + (double)bm * bn * lagom::elem_size(out_dt);
    out->tile_m = (int32_t)bm; out->tile_n = (int32_t)bn; out->tile_k = BK; out->threads = THREADS;
    // the block of tiles an XCD works on at a time under tile_of() (32 compute units per XCD): n tiles in
    // r tile-rows and c tile-columns need r A panels and c B panels between them
    const int64_t total = tm * tn;
    int64_t n, rows, cols;
    if (total % 8 == 0) {
        n = total / 8 < 32 ? total / 8 : 32;
        rows = tm < 8 ? tm : 8;
        if (rows > n) rows = n;
        cols = (n + rows - 1) / rows;
    } else {   // ids are not remapped: an XCD holds every eighth tile of the column-of-8 order
        n = (total + 7) / 8 < 32 ? (total + 7) / 8 : 32;
        rows = 1;
        cols = n;
    }
    out->d_bytes_past_l2 = ((double)rows * bm + (double)cols * bn) * (double)K * 2.0 / (double)n +
                           (double)bm * bn * lagom::elem_size(out_dt);
    return LAGOM_OK;
}

extern "C" int lagom_gemm(const void* A, const void* B, void* C, int64_t M, int64_t N, int64_t K,
                          int b_is_nk, lagom_dtype out_dt, void* hip_stream) {
    if (int rc = lagom::check_gemm_args(A, B, C, M, N, K, out_dt)) return rc;
    if (!b_is_nk && (N % 8)) return lagom::fail(LAGOM_EINVAL, "B stored [K,N] needs N to be a multiple of 8");
    const Tiling tiling = choose_tiling(M, N, K);
    if (tiling != TILE_256x256) {
        const int bm = tiling == TILE_128x128 ? SBM : MBM;
        GemmArgs a{static_cast<const uint16_t*>(A), static_cast<const uint16_t*>(B), C, M, N, K,
                   (int32_t)((M + bm - 1) / bm), (int32_t)((N + SBN - 1) / SBN)};
        const dim3 grid((unsigned)(a.tiles_m * a.tiles_n));
        hipStream_t st = static_cast<hipStream_t>(hip_stream);
        const bool bf = out_dt == LAGOM_BF16;
        const bool tail = K % BK != 0;
        int rc;
#define LAGOM_PICK(NAME) (bf ? launch_fast<NAME<true>>(a, grid, st) : launch_fast<NAME<false>>(a, grid, st))
        if (tiling == TILE_128x128) {
            if (b_is_nk) rc = tail ? LAGOM_PICK(gemm_bf16_nk128_tail_kernel) : LAGOM_PICK(gemm_bf16_nk128_kernel);
            else rc = tail ? LAGOM_PICK(gemm_bf16_kn128_tail_kernel) : LAGOM_PICK(gemm_bf16_kn128_kernel);
        } else {
            if (b_is_nk) rc = tail ? LAGOM_PICK(gemm_bf16_nk256x128_tail_kernel) : LAGOM_PICK(gemm_bf16_nk256x128_kernel);
            else rc = tail ? LAGOM_PICK(gemm_bf16_kn256x128_tail_kernel) : LAGOM_PICK(gemm_bf16_kn256x128_kernel);
        }
#undef LAGOM_PICK
        if (rc) return rc;
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return lagom::fail(LAGOM_EHIP, "gemm launch: %s", hipGetErrorString(e));
        return LAGOM_OK;
    }
    GemmArgs a{static_cast<const uint16_t*>(A), static_cast<const uint16_t*>(B), C, M, N, K,
               (int32_t)((M + BM - 1) / BM), (int32_t)((N + BN - 1) / BN)};
    const int64_t tiles = (int64_t)a.tiles_m * a.tiles_n;
    if (tiles > (1 << 30)) return lagom::fail(LAGOM_EINVAL, "too many tiles");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const dim3 grid((unsigned)tiles), block(THREADS);
    const bool bf = out_dt == LAGOM_BF16;
    const bool fast = K >= BK && K <= FAST_MAX_K && (b_is_nk || N <= FAST_MAX_N_KN);
    if (fast) {
        int rc;
        if (K % BK == 0) {
            if (b_is_nk) rc = bf ? launch_fast<gemm_bf16_nk_kernel<true>>(a, grid, st) : launch_fast<gemm_bf16_nk_kernel<false>>(a, grid, st);
            else rc = bf ? launch_fast<gemm_bf16_kn_kernel<true>>(a, grid, st) : launch_fast<gemm_bf16_kn_kernel<false>>(a, grid, st);
        } else {
            if (b_is_nk) rc = bf ? launch_fast<gemm_bf16_nk_tail_kernel<true>>(a, grid, st) : launch_fast<gemm_bf16_nk_tail_kernel<false>>(a, grid, st);
            else rc = bf ? launch_fast<gemm_bf16_kn_tail_kernel<true>>(a, grid, st) : launch_fast<gemm_bf16_kn_tail_kernel<false>>(a, grid, st);
        }
        if (rc) return rc;
    } else if (b_is_nk) {
        if (bf) hipLaunchKernelGGL((gemm_bf16_general_kernel<true, true>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((gemm_bf16_general_kernel<true, false>), grid, block, 0, st, a);
    } else {
        if (bf) hipLaunchKernelGGL((gemm_bf16_general_kernel<false, true>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((gemm_bf16_general_kernel<false, false>), grid, block, 0, st, a);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return lagom::fail(LAGOM_EHIP, "gemm launch: %s", hipGetErrorString(e));
    return LAGOM_OK;
}
