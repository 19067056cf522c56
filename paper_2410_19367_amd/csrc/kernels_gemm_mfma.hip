// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_16x16x32_bf16 in the 256 x 256 tiles and in the
// forward / data-gradient form of the smaller ones, v_mfma_f32_32x32x16_bf16 elsewhere; fp32
// accumulation) for the
// three shapes of a linear layer: forward Y = X W (+b)(+res), dgrad dX = dY W^T, wgrad dW += X^T dY.
//
// A block computes a BM x BN tile of C, stepping over K in slices of BK = 64.  Each slice of
// op(A) and op(B) sits in LDS as 16-byte chunks with no reshaping:
//   * an operand whose contraction index is contiguous in memory ("k-major": X, dY in dgrad,
//     W in dgrad, the transposed weight copies the forward uses) is stored as [row][64 k] and read
//     back with one ds_read_b128 per fragment;
//   * an operand whose row index is contiguous ("r-major": X^T and dY in wgrad) is stored as
//     [k][rows] and read back with the LDS transpose read ds_read_b64_tr_b16, which hands each
//     lane four consecutive k of one row.
// Both layouts XOR-swizzle the chunk index so fragment reads spread over all LDS banks.
// Two kernels: gemm_mfma_kernel stages slices through registers with predication (ragged shapes);
// gemm_dma_kernel (further down) loads them straight into LDS and carries the fused epilogues,
// split-K and multi-segment contractions.  Slices land in LDS while earlier ones feed the MFMAs,
// one barrier per slice: two LDS stages in gemm_mfma_kernel and in the large tiles of
// gemm_dma_kernel, three in its 128 x 128 forward / data-gradient form, a ring of five half-slices
// in its weight-gradient form.
#include <cstdlib>
#include <type_traits>

#include <atomic>

#include "bp_kernels.h"
#include "bp_device.h"

namespace bp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 64;

// ---- LDS layouts (byte offsets inside one operand tile)
// k-major tile [R][64]: 128 bytes per row, chunk c (8 elements) of a row stored at c ^ ((row>>1)&7)
__device__ __forceinline__ int kmajor_off(int row, int chunk) {
    return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4);
}
// r-major tile [64][R]: 2R bytes per k-row, 16-byte chunk c stored at c ^ rmajor_swz(k).  A transpose
// read touches 64 contiguous bytes in each of four consecutive k-rows; the XOR puts those four
// pieces into different 64-byte bank groups.  With R a multiple of 128 the rows start 0 mod 256
// bytes apart (shift by 0/64/128/192 bytes); with R = 192 they alternate 0/128, so rows 2 and 3
// only need a 64-byte shift, which also keeps the XOR inside the row's 24 chunks.
// (The 16x16x32 MFMA shape reads k-rows k .. k+3 and k+8 .. k+11 in one pass of 32 lanes: bit 3 of k
// moves a piece by another 32 bytes.)
template <int R> __device__ __forceinline__ int rmajor_swz(int k) {
    return R % 128 == 0 ? (((k & 3) << 2) | (((k >> 3) & 1) << 1)) : (((k >> 1) & 1) << 2);
}
template <int R>
__device__ __forceinline__ int rmajor_off(int k, int chunk) {
    return k * (2 * R) + ((chunk ^ rmajor_swz<R>(k)) << 4);
}

template <int R> constexpr int tile_bytes() { return R * BK * 2; }

// ---- global -> registers -> LDS for one operand slice.
// NT threads copy R*8 chunks of 16 bytes; CH = chunks per thread.
template <int R, int NT, bool RMAJOR, bool RAGGED>
struct TileLoader {
    static constexpr int CH = R * 8 / NT;
    u32x4 regs[CH];

    // rows_valid: number of valid rows of this tile (M or N remainder); k_valid: valid k in slice
    __device__ __forceinline__ void load(const bf16_t* __restrict__ base, int ld, int rows_valid,
                                         int k_valid) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int q = threadIdx.x + i * NT;
            int row, k;
            if (RMAJOR) { k = q / (R / 8); row = (q % (R / 8)) * 8; }
            else { row = q >> 3; k = (q & 7) * 8; }
            const bf16_t* p = RMAJOR ? base + (size_t)k * ld + row : base + (size_t)row * ld + k;
            if (RAGGED) {
                // chunks are 8 elements along the contiguous axis; shapes are multiples of 8 there
                const bool ok = row < rows_valid && k < k_valid;
                const u32x4 zero = {0u, 0u, 0u, 0u};
                regs[i] = ok ? *reinterpret_cast<const u32x4*>(p) : zero;
            } else {
                regs[i] = *reinterpret_cast<const u32x4*>(p);
            }
        }
    }
    __device__ __forceinline__ void store(char* lds) const {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int q = threadIdx.x + i * NT;
            int off;
            if (RMAJOR) off = rmajor_off<R>(q / (R / 8), q % (R / 8));
            else off = kmajor_off(q >> 3, q & 7);
            *reinterpret_cast<u32x4*>(lds + off) = regs[i];
        }
    }
};

// ---- fragment read: 8 consecutive k (k16 step kk, half h = lane/32) of row (row0 + lane%32)
template <int R, bool RMAJOR>
__device__ __forceinline__ bf16x8 read_frag(const char* lds, int row0, int kk, int lane) {
    const int h = lane >> 5;
    if (!RMAJOR) {
        const int row = row0 + (lane & 31);
        return *reinterpret_cast<const bf16x8*>(lds + kmajor_off(row, kk * 2 + h));
    } else {
        // transpose read: within a group of 16 lanes, lane i receives element (i%4) of the four
        // 8-byte rows addressed by lanes r*4 + i/4 (r = 0..3).  Lane j = 4r + q therefore points
        // at k-row (k0 + r), elements [col0 + 4q, col0 + 4q + 4), and lane i ends up with
        // k0..k0+3 of column col0 + i.
        const int i = lane & 15, g2 = (lane >> 4) & 1;
        const int r = i >> 2, q = i & 3;
        const int col = row0 + 16 * g2 + 4 * q;       // element index along the r-major row
        const int chunk = col >> 3, byte = (col & 7) * 2;
        const int k0 = kk * 16 + 8 * h;
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (s16x4 __attribute__((address_space(3)))*)(lds + rmajor_off<R>(k0 + r, chunk) + byte));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (s16x4 __attribute__((address_space(3)))*)(lds + rmajor_off<R>(k0 + 4 + r, chunk) + byte));
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, v);
    }
}

// ---- the kernel
// WM x WN waves, each owning a (BM/WM) x (BN/WN) sub-tile made of 32x32 MFMA tiles.
template <int BM, int BN, int WM, int WN, bool A_RMAJOR, bool B_RMAJOR, bool RAGGED>
__global__ __launch_bounds__(WM* WN * 64) void gemm_mfma_kernel(GemmArgs g, int tiles_m, int tiles_n) {
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;   // MFMA tiles per wave
    constexpr int A_BYTES = tile_bytes<BM>(), B_BYTES = tile_bytes<BN>();
    extern __shared__ __attribute__((aligned(16))) char smem[];

    // Blocks are dealt round-robin to the 8 XCDs; give each XCD a contiguous band of tiles so the
    // blocks sharing an L2 also share rows of A, and walk tiles column-first inside the band.
    const int nblk = tiles_m * tiles_n;
    int bid = blockIdx.x;
    if (nblk % 8 == 0) bid = (bid & 7) * (nblk >> 3) + (bid >> 3);
    const int tm = bid / tiles_n, tn = bid % tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / WN, wn = wave % WN;

    const bf16_t* A = (const bf16_t*)g.A;
    const bf16_t* B = (const bf16_t*)g.B;
    // op(A) rows are m; k-major: A[m*lda + k]; r-major (a_t): A[k*lda + m]
    const bf16_t* a_base = A_RMAJOR ? A + m0 : A + (size_t)m0 * g.lda;
    // op(B) rows are n; k-major (b_t): B[n*ldb + k]; r-major: B[k*ldb + n]
    const bf16_t* b_base = B_RMAJOR ? B + n0 : B + (size_t)n0 * g.ldb;
    const size_t a_step = A_RMAJOR ? (size_t)BK * g.lda : BK;
    const size_t b_step = B_RMAJOR ? (size_t)BK * g.ldb : BK;
    const int m_valid = g.M - m0, n_valid = g.N - n0;

    TileLoader<BM, NT, A_RMAJOR, RAGGED> la;
    TileLoader<BN, NT, B_RMAJOR, RAGGED> lb;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nk = (g.K + BK - 1) / BK;
    la.load(a_base, g.lda, m_valid, g.K);
    lb.load(b_base, g.ldb, n_valid, g.K);
    la.store(smem);
    lb.store(smem + A_BYTES);
    if (nk > 1) {
        la.load(a_base + a_step, g.lda, m_valid, g.K - BK);
        lb.load(b_base + b_step, g.ldb, n_valid, g.K - BK);
    }
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        char* sa = smem + cur * (A_BYTES + B_BYTES);
        char* sb = sa + A_BYTES;
        // slice kt+1 (already in registers) goes to the other stage; nobody reads that stage any
        // more: every wave has passed the barrier that ended the previous iteration
        if (kt + 1 < nk) {
            char* na = smem + (cur ^ 1) * (A_BYTES + B_BYTES);
            la.store(na);
            lb.store(na + A_BYTES);
        }
        if (kt + 2 < nk) {
            la.load(a_base + (size_t)(kt + 2) * a_step, g.lda, m_valid, g.K - (kt + 2) * BK);
            lb.load(b_base + (size_t)(kt + 2) * b_step, g.ldb, n_valid, g.K - (kt + 2) * BK);
        }
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = read_frag<BM, A_RMAJOR>(sa, wm * (BM / WM) + i * 32, kk, lane);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = read_frag<BN, B_RMAJOR>(sb, wn * (BN / WN) + j * 32, kk, lane);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // ---- epilogue.  Accumulator v of lane l holds C[8*(v/4) + 4*(l/32) + v%4][l%32] of its tile.
    const int col_l = lane & 31, row_l = 4 * (lane >> 5);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * (BN / WN) + j * 32 + col_l;
        if (RAGGED && n >= g.N) continue;
        const float bias = (!g.accumulate && g.bias) ? g.bias[n] : 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * (BM / WM) + i * 32 + 8 * (v >> 2) + row_l + (v & 3);
                if (RAGGED && m >= g.M) continue;
                const size_t o = (size_t)m * g.ldc + n;
                if (g.accumulate) {
                    float* c = (float*)g.C + o;
                    *c = g.accumulate == 2 ? acc[i][j][v] : *c + acc[i][j][v];
                } else {
                    float r = acc[i][j][v] + bias;
                    if (g.residual) r += (float)((const bf16_t*)g.residual)[o];
                    ((bf16_t*)g.C)[o] = (bf16_t)r;
                }
            }
        }
    }
}

// =====================================================================================
// Second kernel: aligned shapes.  Slices go global -> LDS directly (global_load_lds, 16 bytes per
// lane, one wave instruction fills 1 KiB of consecutive LDS), so no registers or ds_write issue
// slots are spent on staging; NS LDS stages let the loads run NS-1 slices ahead of the MFMAs.
// Because the hardware fixes the LDS position of each lane's 16 bytes, the swizzled layouts
// are produced by choosing which global chunk each lane fetches.
// =====================================================================================

// (a 16-byte fragment read serves 16 lanes = 16 consecutive rows per cycle: the XOR has to give
// those rows 16 different chunk positions modulo the 256-byte bank period)
template <int BKT> __device__ __forceinline__ int kmaj_swz(int row) {
    return BKT == 128 ? (row & 15) : BKT == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3);
}
// byte offset of logical 16-byte chunk c of `row` in a k-major tile [R][BKT]
template <int BKT> __device__ __forceinline__ int kmaj_off(int row, int c) {
    return row * (BKT * 2) + ((c ^ kmaj_swz<BKT>(row)) << 4);
}

// One wave instruction moves 64 x 16 bytes from global memory straight into 1 KiB of consecutive LDS.
// The global address is a buffer descriptor (wave-uniform tile origin) plus a per-lane 32-bit byte
// offset plus a wave-uniform byte offset (the K slice), so issuing a load costs no vector ALU work.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base) {
    // raw buffer, stride 0, no bounds clamp below 4 GiB - 1; dword 3 as for untyped 32-bit data on gfx9
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)0xffffffffu, 0x00020000);
}
__device__ __forceinline__ void dma16(rsrc_t rsrc, uint32_t lane_off, uint32_t slice_off, char* lds_wave_base) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (void __attribute__((address_space(3)))*)lds_wave_base, 16,
                                             (int)lane_off, (int)slice_off, 0, 0);
}

// s_waitcnt with only vmcnt set (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
#define BP_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N) & 15) | (((N) >> 4) << 14) | (7 << 4) | (15 << 8))

// Per-lane byte offsets (relative to the slice base) of the chunks this lane fetches: 32 bits, so
// that the load takes the wave-uniform slice base from scalar registers plus this one vector register.
template <int R, int BKT, int NW, bool RMAJOR>
struct DmaPlan {
    static constexpr int NI = R * BKT / 512 / NW;   // wave instructions per wave per slice
    uint32_t boff[NI];                              // byte offset from the slice base
    __device__ __forceinline__ void init(int wave, int lane, int ld) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int P = (wave + NW * i) * 64 + lane;          // 16-byte position in the tile
            if (RMAJOR) {
                const int krow = P / (R / 8), p = P % (R / 8);
                boff[i] = 2u * (uint32_t)(krow * ld + ((p ^ rmajor_swz<R>(krow)) << 3));
            } else {
                const int row = P / (BKT / 8), p = P % (BKT / 8);
                boff[i] = 2u * (uint32_t)(row * ld + ((p ^ kmaj_swz<BKT>(row)) << 3));
            }
        }
    }
    __device__ __forceinline__ void issue(rsrc_t tile, uint32_t slice_off, char* lds_tile, int wave) const {
#pragma unroll
        for (int i = 0; i < NI; ++i) dma16(tile, boff[i], slice_off, lds_tile + (wave + NW * i) * 1024);
    }
};

template <int R, int BKT, bool RMAJOR>
__device__ __forceinline__ bf16x8 read_frag2(const char* lds, int row0, int kk, int lane) {
    const int h = lane >> 5;
    if (!RMAJOR) {
        return *reinterpret_cast<const bf16x8*>(lds + kmaj_off<BKT>(row0 + (lane & 31), kk * 2 + h));
    } else {
        const int i = lane & 15, g2 = (lane >> 4) & 1;
        const int r = i >> 2, q = i & 3;
        const int col = row0 + 16 * g2 + 4 * q;
        const int chunk = col >> 3, byte = (col & 7) * 2;
        const int k0 = kk * 16 + 8 * h;
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (s16x4 __attribute__((address_space(3)))*)(lds + rmajor_off<R>(k0 + r, chunk) + byte));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (s16x4 __attribute__((address_space(3)))*)(lds + rmajor_off<R>(k0 + 4 + r, chunk) + byte));
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, v);
    }
}

// The same for the 16x16x32 MFMA shape: 8 consecutive k (k32 step kk, quarter lane/16) of row
// (row0 + lane%16).
template <int R, int BKT, bool RMAJOR>
__device__ __forceinline__ bf16x8 read_frag16(const char* lds, int row0, int kk, int lane) {
    const int g4 = lane >> 4;
    if (!RMAJOR) {
        return *reinterpret_cast<const bf16x8*>(lds + kmaj_off<BKT>(row0 + (lane & 15), kk * 4 + g4));
    } else {
        const int i = lane & 15;
        const int r = i >> 2, q = i & 3;
        const int col = row0 + 4 * q;
        const int chunk = col >> 3, byte = (col & 7) * 2;
        const int k0 = kk * 32 + 8 * g4;
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (s16x4 __attribute__((address_space(3)))*)(lds + rmajor_off<R>(k0 + r, chunk) + byte));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (s16x4 __attribute__((address_space(3)))*)(lds + rmajor_off<R>(k0 + 4 + r, chunk) + byte));
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, v);
    }
}

constexpr int rows_per_instr(int lanes_per_row) {
    int r = 1;
    while (2 * r * lanes_per_row <= 64 && 2 * r <= 32) r *= 2;
    return r;
}

// Tile order: each XCD (blocks are dealt round-robin over 8 XCDs) gets a contiguous range of ids,
// walked in groups of 4 tile rows so that concurrent blocks share A rows and B columns.
__device__ __forceinline__ void tile_coords(int t, int tiles_m, int tiles_n, int& tm, int& tn) {
    const int nblk = tiles_m * tiles_n;
    if (nblk % 8 == 0) t = (t & 7) * (nblk >> 3) + (t >> 3);
    constexpr int GM = 4;
    const int per_group = GM * tiles_n;
    const int first_m = (t / per_group) * GM;
    const int gsize = min(tiles_m - first_m, GM);
    tm = first_m + (t % per_group) % gsize;
    tn = (t % per_group) / gsize;
}

// Issue-order groups for one k step of NMFMA MFMAs.  Inside a slice (NLOAD == 0) the step's NREAD
// LDS reads are spread evenly over all its MFMAs, so the LDS sees a steady stream instead of bursts
// from every wave at once.  At a slice boundary the step also carries NLOAD direct-to-LDS loads
// (those write LDS, so the compiler keeps them on their side of the reads next to them in the
// program): with LF == 0 the reads go out in the first half of the step and the loads in the second;
// with LF > 0 the loads come first, one group per MFMA over the first LF MFMAs, and the reads follow
// (the caller then also issues them first in the program).
constexpr int ceil_div(int a, int b) { return (a + b - 1) / b; }
template <int R, int NMFMA, int NREAD, int NLOAD, int LF = 0>
struct SchedRounds {
    static __device__ __forceinline__ void apply() {
        if constexpr (NLOAD > 0 && LF > 0) {
            constexpr int loads = R >= LF ? 0 : ceil_div((R + 1) * NLOAD, LF) - ceil_div(R * NLOAD, LF);
            constexpr int RR = NMFMA - LF;                                       // rounds that carry reads
            constexpr int Q = R - LF;
            constexpr int reads = Q < 0 ? 0 : ceil_div((Q + 1) * NREAD, RR) - ceil_div(Q * NREAD, RR);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                       // 1 MFMA
            if constexpr (loads > 0) __builtin_amdgcn_sched_group_barrier(0x010, loads, 0);   // VMEM
            if constexpr (reads > 0) __builtin_amdgcn_sched_group_barrier(0x100, reads, 0);   // DS reads
        } else {
            constexpr int RR = NLOAD ? (NMFMA / 2 > 0 ? NMFMA / 2 : 1) : NMFMA;      // rounds that carry reads
            constexpr int reads = R >= RR ? 0 : ceil_div((R + 1) * NREAD, RR) - ceil_div(R * NREAD, RR);
            constexpr int LR = NMFMA - RR > 0 ? NMFMA - RR : 1;                      // rounds that carry loads
            constexpr int L = NLOAD ? R - (NMFMA - LR) : -1;
            constexpr int loads = L < 0 ? 0 : ceil_div((L + 1) * NLOAD, LR) - ceil_div(L * NLOAD, LR);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                       // 1 MFMA
            if constexpr (reads > 0) __builtin_amdgcn_sched_group_barrier(0x100, reads, 0);   // DS reads
            if constexpr (loads > 0) __builtin_amdgcn_sched_group_barrier(0x010, loads, 0);   // VMEM
        }
        if constexpr (R + 1 < NMFMA) SchedRounds<R + 1, NMFMA, NREAD, NLOAD, LF>::apply();
    }
};

template <int BM, int BN, int WM, int WN, int BKT, int NS, bool A_RMAJOR, bool B_RMAJOR, bool MI16 = false, bool RING = false>
__global__ __launch_bounds__(WM* WN * 64) void gemm_dma_kernel(GemmArgs g, int tiles_m, int tiles_n, int splits,
                                                               int n_full) {
    constexpr int NW = WM * WN;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int A_BYTES = BM * BKT * 2, B_BYTES = BN * BKT * 2, STAGE = A_BYTES + B_BYTES;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    // Blocks 0 .. n_full-1 compute whole tiles.  The remaining tiles (the tail of the launch, which
    // would occupy only part of the chip) are cut along K: block n_full + j takes slice j / n_tail
    // of tail tile j % n_tail and leaves an fp32 partial for the reduce kernel.
    const int nblk = tiles_m * tiles_n;
    const int n_tail = nblk - n_full;
    const bool is_split = (int)blockIdx.x >= n_full;
    const int sp = is_split ? ((int)blockIdx.x - n_full) / n_tail : 0;
    const int tail_idx = is_split ? ((int)blockIdx.x - n_full) % n_tail : 0;
    const int eff_splits = is_split ? splits : 1;
    int tm, tn;
    tile_coords(is_split ? n_full + tail_idx : (int)blockIdx.x, tiles_m, tiles_n, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform by construction
    const int wm = wave / WN, wn = wave % WN;

    // The contraction runs over g.nseg operand pairs of g.K each; this block owns steps
    // [k_first, k_first + nk) of the concatenation.  (seg, kl) is the position of the next slice
    // to request.
    const int nk_seg = g.K / BKT;
    const int nk_all = nk_seg * g.nseg;
    // K slices of a split tile differ by at most one step: the first nk_all % splits get one more
    const int nk = nk_all / eff_splits + (sp < nk_all % eff_splits ? 1 : 0);
    const int k_first = sp * (nk_all / eff_splits) + min(sp, nk_all % eff_splits);
    // byte step of one K slice inside a segment
    const uint32_t a_step = 2u * (uint32_t)(A_RMAJOR ? BKT * g.lda : BKT);
    const uint32_t b_step = 2u * (uint32_t)(B_RMAJOR ? BKT * g.ldb : BKT);
    auto a_origin = [&](int sgm) {
        const bf16_t* A = (const bf16_t*)(sgm == 0 ? g.A : g.A_more[sgm - 1]);
        return make_rsrc(A_RMAJOR ? A + m0 : A + (size_t)m0 * g.lda);
    };
    auto b_origin = [&](int sgm) {
        const bf16_t* Bp = (const bf16_t*)(sgm == 0 ? g.B : g.B_more[sgm - 1]);
        return make_rsrc(B_RMAJOR ? Bp + n0 : Bp + (size_t)n0 * g.ldb);
    };
    // the next slice to request: segment, slice inside it, tile origins of that segment, byte offsets
    int seg = k_first / nk_seg, kl = k_first % nk_seg;
    rsrc_t a_tile = a_origin(seg), b_tile = b_origin(seg);
    uint32_t a_off = kl * a_step, b_off = kl * b_step;
    int issued = 0;                                     // slices requested so far
    // move on to the next slice, unless the last one has just been requested: then stay on it
    auto advance = [&]() {
        ++issued;
        if (issued >= nk) return;
        a_off += a_step;
        b_off += b_step;
        if (++kl == nk_seg) {
            kl = 0;
            ++seg;
            a_tile = a_origin(seg);
            b_tile = b_origin(seg);
            a_off = b_off = 0;
        }
    };

    DmaPlan<BM, BKT, NW, A_RMAJOR> pa;
    DmaPlan<BN, BKT, NW, B_RMAJOR> pb;
    pa.init(wave, lane, g.lda);
    pb.init(wave, lane, g.ldb);
    constexpr int LPT = decltype(pa)::NI + decltype(pb)::NI;   // loads per slice per wave

    // MI16: the tile is made of 16x16x32 MFMAs instead of 32x32x16 ones, and a "k step" below is 32
    // deep instead of 16.  Per flop that shape reads and writes half as many accumulator registers;
    // under sustained load, where the chip runs against its power limit, a loop of nothing but MFMAs
    // on random operands reaches 1.9 PFLOP/s with it against 1.35 - 1.65 with the 32x32x16 shape
    // (two waves per SIMD; one wave alone cannot issue the 16-cycle instructions back to back).  Inside
    // the stages the 256 x 256 tiles gain 2 % (step time), the weight-gradient form 4 - 6 %; on the
    // 192-wide and the 128 x 128 tiles it made no difference, so those keep the 32x32x16 shape.
    typedef float f32x4acc __attribute__((ext_vector_type(4)));
    constexpr int FM = MI16 ? BM / WM / 16 : TM, FN = MI16 ? BN / WN / 16 : TN;   // fragments per k step
    f32x16 acc[MI16 ? 1 : TM][MI16 ? 1 : TN];
    f32x4acc acc16[MI16 ? FM : 1][MI16 ? FN : 1];
    if constexpr (MI16) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc16[i][j][v] = 0.f;
    } else {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    }

    constexpr int KK = MI16 ? BKT / 32 : BKT / 16;
    static_assert(KK >= 2 && KK % 2 == 0, "a K slice is an even number of k steps");
    static_assert(NS >= 2 && NS <= 5, "2 to 5 LDS stages");
    static_assert((NS - 2) * LPT < 64, "outstanding loads must fit the vmcnt field");
    constexpr int NREAD = (FM * (A_RMAJOR ? 2 : 1) + FN * (B_RMAJOR ? 2 : 1));   // LDS reads per k step
    bf16x8 fa[2][FM], fb[2][FN];
    // program order = issue order of the reads: the fragments the step's first MFMAs need (A row
    // block 0 and every B column block) before the other A row blocks
    auto read_step = [&](const char* sa, int kk, int buf) {
        constexpr int LBK = RING ? 32 : BKT;            // K depth of one LDS tile (ring: slots of 32)
        const char* sb = sa + BM * LBK * 2;
        if constexpr (MI16) {
            fa[buf][0] = read_frag16<BM, LBK, A_RMAJOR>(sa, wm * (BM / WM), kk, lane);
#pragma unroll
            for (int j = 0; j < FN; ++j) fb[buf][j] = read_frag16<BN, LBK, B_RMAJOR>(sb, wn * (BN / WN) + j * 16, kk, lane);
#pragma unroll
            for (int i = 1; i < FM; ++i) fa[buf][i] = read_frag16<BM, LBK, A_RMAJOR>(sa, wm * (BM / WM) + i * 16, kk, lane);
        } else {
        fa[buf][0] = read_frag2<BM, BKT, A_RMAJOR>(sa, wm * (BM / WM), kk, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[buf][j] = read_frag2<BN, BKT, B_RMAJOR>(sb, wn * (BN / WN) + j * 32, kk, lane);
#pragma unroll
        for (int i = 1; i < TM; ++i) fa[buf][i] = read_frag2<BM, BKT, A_RMAJOR>(sa, wm * (BM / WM) + i * 32, kk, lane);
        }
    };
    auto mfma_step = [&](int buf) {
        if constexpr (MI16) {
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc16[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[buf][i], fb[buf][j], acc16[i][j], 0, 0, 0);
        } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);
        }
    };
    // Issue order inside a k16 step, pinned completely (an MFMA left out of the groups could drift
    // across the slice boundary): the LDS reads of the next step spread over the first MFMAs.  At a
    // slice boundary the MFMAs of the slice's last k16 step also carry the direct-to-LDS loads of the
    // slice NS ahead.
    constexpr int NMFMA = FM * FN;
    auto interleave = [&]() { SchedRounds<0, NMFMA, NREAD, 0>::apply(); };
    // Loads first in the barrier's step for the 16x16x32 tiles with both operands contraction-major:
    // that kernel runs at a higher clock than the 32x32x16 one (see above) and waits for its loads at
    // the next barrier (a quarter of a slice's time in a build with cycle-counter stamps), so every
    // cycle they go out earlier counts: +6 - 10 % on the large forward / data-gradient products.  The
    // weight-gradient ring and the 32x32x16 tiles are faster the other way round.
    constexpr int LF = (MI16 && !RING && !A_RMAJOR && !B_RMAJOR) ? (NMFMA / 2 < 8 ? NMFMA / 2 : 8) : 0;
    auto interleave_boundary = [&]() { SchedRounds<0, NMFMA, NREAD, LPT, LF>::apply(); };
    // wait until at most `n` of the most recently requested slices are still on their way
    auto wait_slices = [&](int n) {
        if (NS > 4 && n >= 3) { BP_WAIT_VMCNT(3 * LPT); }
        else if (NS > 3 && n == 2) { BP_WAIT_VMCNT(2 * LPT); }
        else if (NS > 2 && n == 1) { BP_WAIT_VMCNT(1 * LPT); }
        else { BP_WAIT_VMCNT(0); }
    };

    // NS stages: while slice kt feeds the MFMAs, slices kt+1 .. kt+NS-1 are landing or have landed.
    // The barrier between slices sits in front of the *last* k16 step of a slice, whose fragments are
    // already in registers.  Past the barrier the first fragments of the next slice are requested and
    // the loads of slice kt+NS are issued into the stage just freed, in between the MFMAs of that last
    // step, so no wave starts a slice with an empty matrix pipe.
    // The loop body has no branches (the compiler interleaves and counts outstanding reads exactly
    // only inside one basic block): once every slice has been requested the body keeps requesting
    // the last one again (into stages nobody reads any more) and past the last slice it reads
    // fragments nobody uses; the change from one contraction segment to the next happens between
    // runs of the loop.
    if constexpr (RING) {
        // Ring mode (the weight-gradient form): five LDS slots of 32 along K, one k step each (5 x 32 KB
        // for a 256 x 256 tile: the whole LDS), instead of two stages of 64.  An iteration still covers
        // 64 of K with one barrier between its two k steps.  Past the barrier it requests the slot that
        // the iteration after next reads first, into the first slot it has just freed; the second freed
        // slot is requested one k step later, in the next iteration's first step, and has a barrier
        // more to land: the barrier only ever waits for the older of the two requests, and the loads
        // go out in two bursts per iteration instead of one.  Measured on the
        // weight-gradient shapes of the GPT-style stages: +13 % (2048 x 8192 x 16384: 1130 -> 1280
        // TFLOP/s); with both operands contraction-major it is 2 % slower than two stages (a slot of 32
        // along K is then half a cache line per row, and the requests to the L2 double), so those keep
        // them.
        static_assert(!RING || (MI16 && BKT == 64 && NS == 5), "ring mode: 16x16x32 MFMAs, five slots of 32");
        constexpr int SLOT = (BM + BN) * 32 * 2;
        DmaPlan<BM, 32, NW, A_RMAJOR> ra;
        DmaPlan<BN, 32, NW, B_RMAJOR> rb;
        ra.init(wave, lane, g.lda);
        rb.init(wave, lane, g.ldb);
        constexpr int L32 = decltype(ra)::NI + decltype(rb)::NI;    // loads per slot per wave
        const int nq = 2 * nk;                                      // slots this block walks through
        const uint32_t a_step32 = a_step / 2, b_step32 = b_step / 2;
        auto request = [&](int slot) {
            ra.issue(a_tile, a_off, smem + slot * SLOT, wave);
            rb.issue(b_tile, b_off, smem + slot * SLOT + BM * 64, wave);
            // (no branch) past the end the last slot is requested again, into slots nobody reads any more
            ++issued;
            a_off += issued < nq ? a_step32 : 0u;
            b_off += issued < nq ? b_step32 : 0u;
        };
        auto interleave_l = [&]() { SchedRounds<0, NMFMA, NREAD, L32>::apply(); };
        // The requests walk through the contraction segments 32 deep at a time; a segment holds an even
        // number of slots and the loop requests two per iteration, so the change from one segment to
        // the next falls between two runs of the (branch-free) loop, as in the staged loop below.
        const int nq_seg = 2 * nk_seg;
        int kl32 = 2 * kl;                                          // slots requested so far in the current segment
        auto next_segment = [&]() {
            if (issued < nq && kl32 == nq_seg) {
                kl32 = 0;
                ++seg;
                a_tile = a_origin(seg);
                b_tile = b_origin(seg);
                a_off = b_off = 0;
            }
        };
        a_off = (uint32_t)kl32 * a_step32;
        b_off = (uint32_t)kl32 * b_step32;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            request(q);
            ++kl32;
            next_segment();
        }
        BP_WAIT_VMCNT(2 * L32);                                     // slots 0 and 1 have landed
        __builtin_amdgcn_s_barrier();
        read_step(smem, 0, 0);
        int s0 = 0;                                                 // slot of the first half of the current slice
        int late = 4;                                               // slot of the request that has a barrier more to land
        int it = 0;
        while (it < nk) {
            const int run = issued < nq ? min(nk - it, (nq_seg - kl32) / 2) : nk - it;
            for (int r = 0; r < run; ++r) {
                const int s1 = s0 + 1 >= 5 ? s0 - 4 : s0 + 1;
                const int n0 = s0 + 2 >= 5 ? s0 - 3 : s0 + 2;
                read_step(smem + s1 * SLOT, 0, 1);
                request(late);
                mfma_step(0);
                interleave_l();
                __builtin_amdgcn_sched_barrier(0);
                __builtin_amdgcn_s_waitcnt(0xC07F);         // lgkmcnt(0)
                BP_WAIT_VMCNT(L32);                          // only the request just made may still be on its way
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
                read_step(smem + n0 * SLOT, 0, 0);
                request(s0);
                late = s1;
                mfma_step(1);
                interleave_l();
                s0 = n0;
            }
            it += run;
            kl32 += 2 * run;
            next_segment();
        }
    } else {
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) {
        if (s < nk) {
            pa.issue(a_tile, a_off, smem + s * STAGE, wave);
            pb.issue(b_tile, b_off, smem + s * STAGE + A_BYTES, wave);
            advance();
        }
    }
    wait_slices(min(nk, NS - 1) - 1);                   // slice 0 has landed
    __syncthreads();
    if (NS - 1 < nk) {
        pa.issue(a_tile, a_off, smem + (NS - 1) * STAGE, wave);
        pb.issue(b_tile, b_off, smem + (NS - 1) * STAGE + A_BYTES, wave);
        advance();
    }
    read_step(smem, 0, 0);
    int cur = 0;                                        // stage of slice kt
    int kt = 0;
    while (kt < nk) {
        // a run of the loop below never takes the requests across the end of a segment
        const int run = issued < nk ? min(nk - kt, nk_seg - kl) : nk - kt;
        for (int it = 0; it < run; ++it) {
            const char* sa = smem + cur * STAGE;
#pragma unroll
            for (int kk = 0; kk + 1 < KK; ++kk) {
                read_step(sa, kk + 1, (kk + 1) & 1);
                mfma_step(kk & 1);
                interleave();
            }
            // every LDS read of slice kt has returned (the last ones feed the MFMAs below) and this
            // wave's part of slice kt+1 has landed: the barrier publishes that slice and frees the
            // stage of slice kt
            // (a bare s_barrier: __syncthreads() carries a release fence, for which the compiler waits
            // for every outstanding load, those of the slices further ahead included)
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_waitcnt(0xC07F);         // lgkmcnt(0)
            BP_WAIT_VMCNT((NS - 2) * LPT);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            const int nxt = cur + 1 == NS ? 0 : cur + 1;
            if constexpr (LF == 0) read_step(smem + nxt * STAGE, 0, 0);
            char* st = smem + cur * STAGE;
            pa.issue(a_tile, a_off, st, wave);
            pb.issue(b_tile, b_off, st + A_BYTES, wave);
            if constexpr (LF > 0) read_step(smem + nxt * STAGE, 0, 0);
            // (no branch) the offsets stop moving once the last slice has been requested
            ++issued;
            a_off += issued < nk ? a_step : 0u;
            b_off += issued < nk ? b_step : 0u;
            mfma_step((KK - 1) & 1);
            interleave_boundary();
            cur = nxt;
        }
        kt += run;
        kl += run;
        if (issued < nk && kl == nk_seg) {
            kl = 0;
            ++seg;
            a_tile = a_origin(seg);
            b_tile = b_origin(seg);
            a_off = b_off = 0;
        }
    }
    }
    BP_WAIT_VMCNT(0);                                   // the repeated requests too have landed

    // ---- epilogue through LDS.  The accumulators hold one column and 16 scattered rows per
    // lane; writing them out directly costs one narrow store instruction per element.  Each
    // wave instead lays 32 rows of its tile out in its own LDS region and reads them back with
    // 16 bytes per lane, so global stores (and the fp32 read-modify-write of a weight gradient)
    // are full 16-byte accesses over 256-byte row segments.
    __syncthreads();                                    // every wave is done reading the stages
    constexpr int WTN = BN / WN;                        // wave tile width
    constexpr int PITCH = WTN + 8;                      // floats; 4 rows apart = 32 banks apart
    float* ep = (float*)smem + wave * (32 * PITCH);
    const int h = lane >> 5;
    const int n_base = n0 + wn * WTN;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m_base = m0 + wm * (BM / WM) + i * 32;
        // EPI_GELU_BWD: the pre-activation values of this 32-row slab are requested before the
        // accumulators are staged, so their latency overlaps the LDS round trip
        constexpr int ELPR = WTN / 8, ERPI = rows_per_instr(ELPR), ENR = 32 / ERPI;
        u32x4 upre[ENR];
        if (g.epi == EPI_GELU_BWD && !is_split) {
#pragma unroll
            for (int r = 0; r < ENR; ++r) {
                const int row = r * ERPI + lane / ELPR;
                if (ELPR * ERPI < 64 && lane >= ELPR * ERPI) continue;
                upre[r] = *reinterpret_cast<const u32x4*>((const bf16_t*)g.U + (size_t)(m_base + row) * g.ldc +
                                                          n_base + (lane % ELPR) * 8);
            }
        }
        if constexpr (MI16) {
            // lane l holds column l % 16 and rows 4 * (l / 16) .. + 3 of every 16 x 16 tile
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int i2 = 0; i2 < 2; ++i2)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        ep[(16 * i2 + 4 * (lane >> 4) + v) * PITCH + j * 16 + (lane & 15)] = acc16[2 * i + i2][j][v];
        } else {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                ep[(8 * (v >> 2) + 4 * h + (v & 3)) * PITCH + j * 32 + (lane & 31)] = acc[i][j][v];
        }
        // rows per instruction: the largest power of two whose lanes fit in a wave (a 96-wide wave
        // tile leaves a quarter of the lanes idle here)
        if (is_split) {             // fp32 partial of this K slice: [tail tile][slice][BM][BN]
            constexpr int LPR = WTN / 4, RPI = rows_per_instr(LPR);
            const int col = (lane % LPR) * 4;
            float* slab = g.split_ws + ((size_t)tail_idx * splits + sp) * (BM * BN) +
                          (size_t)(wm * (BM / WM) + i * 32) * BN + wn * WTN;
#pragma unroll
            for (int r = 0; r < 32; r += RPI) {
                const int row = r + lane / LPR;
                if (LPR * RPI < 64 && lane >= LPR * RPI) continue;
                *reinterpret_cast<f32x4*>(slab + (size_t)row * BN + col) =
                    *reinterpret_cast<const f32x4*>(ep + row * PITCH + col);
            }
        } else if (g.accumulate) {
            constexpr int LPR = WTN / 4, RPI = rows_per_instr(LPR);   // lanes per row, rows per instruction
            const int col = (lane % LPR) * 4;
#pragma unroll
            for (int r = 0; r < 32; r += RPI) {
                const int row = r + lane / LPR;
                if (LPR * RPI < 64 && lane >= LPR * RPI) continue;
                const f32x4 v = *reinterpret_cast<const f32x4*>(ep + row * PITCH + col);
                f32x4* c = reinterpret_cast<f32x4*>((float*)g.C + (size_t)(m_base + row) * g.ldc + n_base + col);
                if (g.accumulate == 2) *c = v;      // first contribution after a clear: no read
                else *c = *c + v;
            }
        } else {
            constexpr int LPR = WTN / 8, RPI = rows_per_instr(LPR);
            const int col = (lane % LPR) * 8;
            float bias[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) bias[e] = g.bias ? g.bias[n_base + col + e] : 0.f;
            float csum[8] = {0, 0, 0, 0, 0, 0, 0, 0};      // EPI_GELU_BWD: column sums of this slab
#pragma unroll
            for (int r = 0; r < 32; r += RPI) {
                const int row = r + lane / LPR;
                if (LPR * RPI < 64 && lane >= LPR * RPI) continue;
                const f32x4 v0 = *reinterpret_cast<const f32x4*>(ep + row * PITCH + col);
                const f32x4 v1 = *reinterpret_cast<const f32x4*>(ep + row * PITCH + col + 4);
                float o[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
                const size_t off = (size_t)(m_base + row) * g.ldc + n_base + col;
                if (g.epi == EPI_GELU_FWD) {
                    float act[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) act[e] = gelu_value(o[e] + bias[e]);
                    store8((bf16_t*)g.C + off, o);
                    store8((bf16_t*)g.C2 + off, act);
                } else if (g.epi == EPI_GELU_BWD) {
                    const u32x4 ur = upre[r / RPI];
                    const float u8[8] = {__uint_as_float(ur[0] << 16), __uint_as_float(ur[0] & 0xffff0000u),
                                         __uint_as_float(ur[1] << 16), __uint_as_float(ur[1] & 0xffff0000u),
                                         __uint_as_float(ur[2] << 16), __uint_as_float(ur[2] & 0xffff0000u),
                                         __uint_as_float(ur[3] << 16), __uint_as_float(ur[3] & 0xffff0000u)};
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        o[e] *= gelu_slope(u8[e] + bias[e]);
                        csum[e] += o[e];
                    }
                    store8((bf16_t*)g.C + off, o);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] += bias[e];
                    if (g.residual) {
                        float rs[8];
                        load8((const bf16_t*)g.residual + off, rs);
#pragma unroll
                        for (int e = 0; e < 8; ++e) o[e] += rs[e];
                    }
                    store8((bf16_t*)g.C + off, o);
                }
            }
            if (g.epi == EPI_GELU_BWD) {
                // lanes l, l + LPR, l + 2 LPR, ... hold the same columns (LPR is a power of two here)
#pragma unroll
                for (int e = 0; e < 8; ++e)
#pragma unroll
                    for (int o2 = LPR; o2 < 64; o2 <<= 1) csum[e] += __shfl_xor(csum[e], o2, 64);
                if (lane < LPR) store8(g.colpart + (size_t)(m_base >> 5) * g.N + n_base + col, csum);
            }
        }
    }
}

// ---- host-side selection
template <int BM, int BN, int WM, int WN, bool RAGGED>
static hipError_t launch_cfg(const GemmArgs& g, hipStream_t s) {
    const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    const dim3 grid(tiles_m * tiles_n), block(WM * WN * 64);
    const size_t smem = 2 * (size_t)(tile_bytes<BM>() + tile_bytes<BN>());
#define BP_GEMM_LAUNCH(AR, BR)                                                                   \
    do {                                                                                         \
        auto kern = gemm_mfma_kernel<BM, BN, WM, WN, AR, BR, RAGGED>;                            \
        static std::atomic<bool> attr_set{false};   /* once per instantiation; host threads may race */ \
        if (smem > 64 * 1024 && !attr_set.load(std::memory_order_acquire)) {                                                     \
            hipError_t e = hipFuncSetAttribute((const void*)kern,                                \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem); \
            if (e != hipSuccess) return e;                                                       \
            attr_set.store(true, std::memory_order_release);                                     \
        }                                                                                        \
        hipLaunchKernelGGL(kern, grid, block, smem, s, g, tiles_m, tiles_n);                     \
    } while (0)
    if (!g.a_t && !g.b_t) BP_GEMM_LAUNCH(false, true);        // forward: X k-major, W[K,N] r-major
    else if (!g.a_t && g.b_t) BP_GEMM_LAUNCH(false, false);   // dgrad: dY k-major, W[n][k] k-major
    else if (g.a_t && !g.b_t) BP_GEMM_LAUNCH(true, true);     // wgrad: X^T r-major, dY r-major
    else BP_GEMM_LAUNCH(true, false);
#undef BP_GEMM_LAUNCH
    return hipGetLastError();
}

// Sum the K-slice partials of the tail tiles in slice order and apply the epilogue; 8 outputs per
// thread, BM * BN / 2048 blocks per tile.
template <int BM, int BN>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(GemmArgs g, int splits, int tiles_m, int tiles_n,
                                                            int n_full) {
    constexpr int BPT = BM * BN / 2048;                 // blocks per tile
    const int tail_idx = blockIdx.x / BPT;
    int tm, tn;
    tile_coords(n_full + tail_idx, tiles_m, tiles_n, tm, tn);
    const int v = (blockIdx.x % BPT) * 256 + threadIdx.x;      // 8-element vector inside the tile
    const int r = v / (BN / 8), c = (v % (BN / 8)) * 8;
    const int m = tm * BM + r, n = tn * BN + c;
    const float* slab = g.split_ws + (size_t)tail_idx * splits * (BM * BN) + (size_t)r * BN + c;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int sp = 0; sp < splits; ++sp) {
        float p[8];
        load8(slab + (size_t)sp * (BM * BN), p);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] += p[i];
    }
    const size_t off = (size_t)m * g.ldc + n;
    if (g.accumulate == 2) {
        store8((float*)g.C + off, acc);
    } else if (g.accumulate) {
        float cc[8];
        load8((const float*)g.C + off, cc);
#pragma unroll
        for (int i = 0; i < 8; ++i) cc[i] += acc[i];
        store8((float*)g.C + off, cc);
    } else {
        if (g.bias) {
            float bv[8];
            load8(g.bias + n, bv);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] += bv[i];
        }
        if (g.residual) {
            float rs[8];
            load8((const bf16_t*)g.residual + off, rs);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] += rs[i];
        }
        store8((bf16_t*)g.C + off, acc);
    }
}

template <int BM, int BN, int WM, int WN, int NS, int BKT = 64, bool MI16 = false, bool RING = false>
static hipError_t launch_dma(const GemmArgs& g, hipStream_t s, int splits = 1, int n_full = -1) {
    const int tiles_m = g.M / BM, tiles_n = g.N / BN;
    const int nblk = tiles_m * tiles_n;
    if (splits <= 1) { splits = 1; n_full = nblk; }
    else if (n_full < 0) n_full = 0;                    // every tile is cut along K
    const int n_tail = nblk - n_full;
    const dim3 grid(n_full + n_tail * splits), block(WM * WN * 64);
    const size_t stages = RING ? (size_t)5 * (BM + BN) * 32 * 2 : (size_t)NS * (BM + BN) * BKT * 2;
    const size_t epilogue = (size_t)WM * WN * 32 * (BN / WN + 8) * sizeof(float);
    const size_t smem = stages > epilogue ? stages : epilogue;
#define BP_GEMM_LAUNCH(AR, BR)                                                                   \
    do {                                                                                         \
        auto kern = gemm_dma_kernel<BM, BN, WM, WN, BKT, NS, AR, BR, MI16, RING>;                         \
        static std::atomic<bool> attr_set{false};   /* once per instantiation; host threads may race */ \
        if (smem > 64 * 1024 && !attr_set.load(std::memory_order_acquire)) {                                                     \
            hipError_t e = hipFuncSetAttribute((const void*)kern,                                \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem); \
            if (e != hipSuccess) return e;                                                       \
            attr_set.store(true, std::memory_order_release);                                     \
        }                                                                                        \
        hipLaunchKernelGGL(kern, grid, block, smem, s, g, tiles_m, tiles_n, splits, n_full);     \
    } while (0)
    if (!g.a_t && !g.b_t) BP_GEMM_LAUNCH(false, true);
    else if (!g.a_t && g.b_t) BP_GEMM_LAUNCH(false, false);
    else if (g.a_t && !g.b_t) BP_GEMM_LAUNCH(true, true);
    else BP_GEMM_LAUNCH(true, false);
#undef BP_GEMM_LAUNCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n_tail == 0) return e;
    hipLaunchKernelGGL((splitk_reduce_kernel<BM, BN>), dim3((unsigned)(n_tail * (BM * BN / 2048))), dim3(256), 0, s,
                       g, splits, tiles_m, tiles_n, n_full);
    return hipGetLastError();
}

bool gemm_mfma_supported(const GemmArgs& g) {
    auto al16 = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
    if (g.K % 8 || g.lda % 8 || g.ldb % 8) return false;
    if (!al16(g.A) || !al16(g.B)) return false;
    for (int i = 0; i + 1 < g.nseg; ++i)
        if (!al16(g.A_more[i]) || !al16(g.B_more[i])) return false;
    // r-major operands are read in 8-element chunks along their row index
    if (g.a_t && g.M % 8) return false;
    if (!g.b_t && g.N % 8) return false;
    return true;
}

static bool dma_path_ok(const GemmArgs& g) {
    auto al16 = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
    bool ok = g.M % 128 == 0 && g.N % 128 == 0 && g.K % BK == 0 && g.ldc % 8 == 0 && al16(g.C) &&
              (!g.residual || al16(g.residual));
    for (int i = 0; i + 1 < g.nseg; ++i) ok = ok && al16(g.A_more[i]) && al16(g.B_more[i]);
    return ok;
}

bool gemm_can_fuse_epilogue(int dtype, const GemmArgs& g) {
    auto al16 = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
    if (dtype != BF16 || !gemm_mfma_supported(g) || !dma_path_ok(g)) return false;
    if (g.accumulate || g.residual || g.nseg != 1 || !g.bias) return false;
    if (g.epi == EPI_GELU_FWD) return g.C2 && al16(g.C2);
    if (g.epi == EPI_GELU_BWD) return g.U && al16(g.U) && g.colpart && al16(g.colpart) && g.N % 8 == 0;
    return false;
}

static int cu_count() {
    static std::atomic<int> cached{0};
    int n = cached.load(std::memory_order_relaxed);
    if (!n) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cached.store(n, std::memory_order_relaxed);
    }
    return n;
}

hipError_t launch_gemm_mfma(const GemmArgs& g, hipStream_t s) {
    auto al16 = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
    const bool aligned128 = dma_path_ok(g);
    if (g.epi != EPI_NONE && !gemm_can_fuse_epilogue(BF16, g)) return hipErrorInvalidValue;
    if (!aligned128) {
        if (g.nseg == 1) return launch_cfg<128, 128, 2, 2, true>(g, s);
        return launch_gemm_per_segment(g, s, [](const GemmArgs& h, hipStream_t st) {
            return launch_cfg<128, 128, 2, 2, true>(h, st);
        });
    }
    const int ncu = cu_count();
    const long k_total = (long)g.K * g.nseg;
    const long most = 3L * ncu / 4;       // a launch with at least this many blocks is taken to fill the chip
    // 256 x 256 tiles (8 waves) once they fill at least three quarters of the CUs
    const bool aligned256 = g.M % 256 == 0 && g.N % 256 == 0;
    const long t256 = aligned256 ? (long)(g.M / 256) * (g.N / 256) : 0;
    // 256 x 192 tiles when they fill the CUs better: e.g. N = 6144 gives 24 columns of 256 (192 tiles
    // for M = 2048, a quarter of the CUs idle) but 32 columns of 192 (256 tiles)
    auto fill = [&](long t) { return t <= 0 ? 0.0 : (double)t / (double)(((t + ncu - 1) / ncu) * ncu); };
    const long t192 = (g.M % 256 == 0 && g.N % 192 == 0) ? (long)(g.M / 256) * (g.N / 192) : 0;
    // (the fused GELU-backward epilogue folds column sums over power-of-two lane groups: not 96 wide)
    // The 192-wide tile has fewer MFMAs per LDS read and per barrier: measured against the 256-wide
    // one at equal fill it runs at about 0.85 of its rate for weight gradients with a long contraction
    // (both operands through the transpose path, no ring) and for the forward / data-gradient form
    // (2048 x 6144 x 2048: 44.5 us against 46.0 us on three quarters of the CUs; 4096 x 15360 x 5120:
    // 543 us against 494 us at a fill of 0.94), else within 5 %.
    const bool nt = !g.a_t && g.b_t;
    const double rate192 = ((g.a_t && !g.b_t && (long)g.K * g.nseg >= 4096) || nt) ? 0.85 : 0.95;
    if (g.epi == EPI_NONE && t192 >= most && rate192 * fill(t192) > fill(t256)) {
        if (nt) return launch_dma<256, 192, 2, 4, 2, 64, true>(g, s);
        return launch_dma<256, 192, 4, 2, 2>(g, s);
    }
    // How many K slices the last, partly filled round of 256 x 256 tiles is cut into so that it fills
    // the chip too (at most 4, each at least 1024 deep so that the fp32 partials stay a small part of
    // the traffic; the slices need not be equal).  With fewer tiles than CUs this is plain split-K.
    auto tail_splits = [&](long tail) {
        int splits = tail > 0 ? (int)(ncu / tail) : 1;
        if (splits > 4) splits = 4;
        while (splits > 1 && (k_total / splits < 1024 || (size_t)splits * tail * 65536 > g.split_ws_elems)) --splits;
        return splits;
    };
    if (t256 >= most) {
        const long full = (t256 / ncu) * ncu, tail = t256 - full;
        const int splits =
            (g.split_ws && g.epi == EPI_NONE && tail < most) ? tail_splits(tail) : 1;
        if (g.a_t && !g.b_t) {      // weight gradients: the five-slot ring
            if (splits > 1) return launch_dma<256, 256, 2, 4, 5, 64, true, true>(g, s, splits, (int)full);
            return launch_dma<256, 256, 2, 4, 5, 64, true, true>(g, s);
        }
        if (splits > 1) return launch_dma<256, 256, 2, 4, 2, 64, true>(g, s, splits, (int)full);
        return launch_dma<256, 256, 2, 4, 2, 64, true>(g, s);
    }
    // Too few 256 x 256 tiles to fill the chip.  Up to a contraction depth of 4096, 128 x 128 tiles
    // that do fill it win over large tiles cut along K: one launch, no fp32 partials (inside the
    // BERT-style stage, 4096 x 1024 x 3072: 41.7 us against 48.6 us).  In the forward / data-gradient
    // form, whose small-tile kernel runs three LDS stages, this holds up to a depth of 8192 when the
    // small tiles fill whole rounds (inside the GPT-style stage, 2048 x 2048 x 8192: 72.7 us against
    // 77.0 us with the partials; but 2048 x 2560 x 7680, 320 tiles on 256 CUs, loses).  Deeper than
    // that, or with a partly filled round, the small tiles lose: they move twice the operand bytes
    // per flop, and inside a layer those come from HBM, not from a warm cache (2048 x 2560 x 10240:
    // 229 us against 115 us).
    // Not for weight gradients either: with both operands read through the transpose path the small
    // tiles lose more than the partials cost (2560 x 2560 x 16384: 334 us against 272 us).
    const long t128 = (long)(g.M / 128) * (g.N / 128);
    const bool small_fill = t128 >= most && (k_total <= 4096 || (nt && k_total <= 8192 && fill(t128) >= 0.95));
    if (small_fill && !(g.a_t && !g.b_t)) {
        if (nt) return launch_dma<128, 128, 2, 4, 3, 64, true>(g, s);
        if (g.K % 128 == 0) return launch_dma<128, 128, 2, 4, 2, 128>(g, s);
        return launch_dma<128, 128, 2, 4, 2>(g, s);
    }
    // Fewer tiles than that but a long K: 256 x 256 tiles on K slices keep the operand traffic per
    // flop at the large-tile level (128 x 128 tiles move twice the operand bytes per flop).
    if (t256 > 0 && g.split_ws && g.epi == EPI_NONE) {
        const int splits = tail_splits(t256);
        if (splits > 1 && t256 * splits * 8 >= 5L * ncu) {
            if (g.a_t && !g.b_t) return launch_dma<256, 256, 2, 4, 5, 64, true, true>(g, s, splits, 0);
            return launch_dma<256, 256, 2, 4, 2, 64, true>(g, s, splits, 0);
        }
    }
    // Small outputs (128 x 128 tiles on fewer than three quarters of the CUs) with a long K: the same split, on the small
    // tiles (slices at least 1024 deep: below that the second kernel costs what the split gains)
    if (g.split_ws && g.epi == EPI_NONE) {
        const int bk = g.K % 128 == 0 ? 128 : BK;
        int splits = (int)(ncu / t128);
        if (splits > 4) splits = 4;
        while (splits > 1 && (k_total / splits < 1024 || (size_t)splits * g.M * g.N > g.split_ws_elems)) --splits;
        if (splits > 1 && nt) return launch_dma<128, 128, 2, 4, 3, 64, true>(g, s, splits, 0);
        if (splits > 1 && bk == 128) return launch_dma<128, 128, 2, 4, 2, 128>(g, s, splits, 0);
        if (splits > 1) return launch_dma<128, 128, 2, 4, 2>(g, s, splits, 0);
    }
    // 8 waves (2 per SIMD) hide the LDS and load latencies better than 4 on these small tiles.
    // Forward / data-gradient form: 16x16x32 MFMAs and loads first, as on the large tiles, and three
    // stages of 64 along K (96 KB), so that a slice has two barriers to land (against two stages of
    // 128: 2048^3 20.7 us against 21.9 us, 2048 x 2048 x 8192 63.7 us against 67.9 us, 1024 x 1024 x
    // 4096 27.9 us against 31.8 us).  The other forms: slices of 128 along K (two stages of 64 KB),
    // which halve the number of barriers per MFMA.
    if (nt) return launch_dma<128, 128, 2, 4, 3, 64, true>(g, s);
    if (g.K % 128 == 0) return launch_dma<128, 128, 2, 4, 2, 128>(g, s);
    return launch_dma<128, 128, 2, 4, 2>(g, s);
}

}  // namespace bp
