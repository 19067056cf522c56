// Fused attention on the gfx950 matrix cores (bf16 inputs, fp32 softmax and accumulation):
// forward with online softmax, and the backward as two deterministic kernels (dQ; dK and dV).
//
// All three kernels stream [64 rows][D] tiles of the packed qkv / dctx tensors through LDS with
// direct global->LDS loads and never materialise an S x S matrix.  Scores are produced
// transposed where that keeps the softmax row of a query inside one lane:
//   forward, dQ :  S^T[key][q] = K Q^T      lane <-> query, registers <-> keys
//   dK, dV      :  S  [q][key] = Q K^T      lane <-> key,   registers <-> queries
// In both cases the probabilities leave the MFMA accumulators as the B operand of the next
// product (the contraction index is the accumulator's row index), so P never goes through LDS.
// The accumulator rows a lane holds come in groups of four consecutive indices, which is exactly
// what the LDS transpose read (ds_read_b64_tr_b16) returns, so the A operands of those second
// products (V^T, K^T, dO^T, Q^T) are read straight from the row-major tiles.
//
// One swizzle serves plain 16-byte fragment reads and transpose reads of the same tile:
// chunk c of row r is stored at c ^ f(r), f chosen so that 16 consecutive rows (plain reads) and
// 4 consecutive rows x 64 bytes (transpose reads) both cover all banks.
#include <atomic>

#include "bp_kernels.h"
#include "bp_device.h"

namespace bp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define BP_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N) & 15) | (((N) >> 4) << 14) | (7 << 4) | (15 << 8))

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// bare v_exp_f32: arguments here are <= 8 and anything below -126 may flush to zero
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Head dimensions below the tile width D (any multiple of 8: 40 -> 64, 96 -> 128): the tile columns
// at and beyond the real width dr are filled from this chunk of zeros and the register fragments
// get zeros there, so the padded part contributes nothing; products that only touch padded columns
// are skipped, and padded output columns are never stored.
__device__ __attribute__((aligned(16))) unsigned int g_zero_chunk[4] = {0u, 0u, 0u, 0u};

// 8 consecutive elements of a row starting at column `col`, zeros at and beyond column dr
__device__ __forceinline__ bf16x8 load_frag(const bf16_t* row, int col, int dr) {
    bf16x8 z;
#pragma unroll
    for (int e = 0; e < 8; ++e) z[e] = (bf16_t)0.f;
    return col < dr ? *reinterpret_cast<const bf16x8*>(row + col) : z;
}

// ---- tile layout: [rows][D] bf16, 16-byte chunks XOR-swizzled by row
template <int D> __device__ __forceinline__ int swz(int row) {
    return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3))
                    : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
}
template <int D> __device__ __forceinline__ int tile_off(int row, int chunk) {
    return row * (D * 2) + ((chunk ^ swz<D>(row)) << 4);
}

// Direct global->LDS copy of a [64][D] tile by NW waves.  Which 16-byte chunk a lane fetches
// depends only on its position, so the per-lane source offsets are computed once per kernel and a
// step only adds the tile's base address (the sequence length is a multiple of 64: every tile
// lies inside its tensor).  dr is the real row width; with PAD, chunks beyond it come from zeros.
template <int D, int NW, bool PAD>
struct TilePlan {
    static constexpr int CPR = D / 8;              // chunks per row
    static constexpr int NI = 64 * CPR / 64 / NW;  // wave instructions per wave
    static constexpr int ROWSTEP = NW * 64 / CPR;  // rows between a lane's consecutive chunks: a multiple
                                                   // of 16, the period of the swizzle, so the column stays
    int off0;                                      // element offset of the first chunk; < 0: padded column
    int ld;                                        // row pitch in elements (wave-uniform)
    __device__ __forceinline__ void init(int wave, int lane, int ld_, int dr) {
        const int P = wave * 64 + lane;
        const int row = P / CPR;
        const int c = (P % CPR) ^ swz<D>(row);
        ld = ld_;
        off0 = (!PAD || c * 8 < dr) ? row * ld + c * 8 : -1;
    }
    // gbase points at (row 0, col 0) of the tile
    __device__ __forceinline__ void issue(const bf16_t* gbase, char* lds, int wave) const {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const bf16_t* src = (!PAD || off0 >= 0) ? gbase + (size_t)i * ROWSTEP * ld + off0
                                                    : (const bf16_t*)g_zero_chunk;
            __builtin_amdgcn_global_load_lds(
                (const void __attribute__((address_space(1)))*)src,
                (void __attribute__((address_space(3)))*)(lds + (wave + NW * i) * 1024), 16, 0, 0);
        }
    }
};

// plain fragment: 8 consecutive columns (k16 step s, half h) of row (row0 + lane%32)
template <int D>
__device__ __forceinline__ bf16x8 frag_rows(const char* lds, int row0, int s, int lane) {
    return *reinterpret_cast<const bf16x8*>(lds + tile_off<D>(row0 + (lane & 31), 2 * s + (lane >> 5)));
}
// transposed fragment for a product whose contraction runs over the tile's rows: lane gets, for
// column (col0 + lane%32), the rows {r0 + 4h .. +3} and {r0 + 8 + 4h .. +3} (h = lane/32): the
// row order in which a 32x32 accumulator hands its 16 rows to the next MFMA.
template <int D>
__device__ __forceinline__ bf16x8 frag_cols(const char* lds, int r0, int col0, int lane) {
    const int i = lane & 15, g2 = (lane >> 4) & 1, h = lane >> 5;
    const int col = col0 + 16 * g2 + 4 * (i & 3);
    const int chunk = col >> 3, byte = (col & 7) * 2;
    const int ra = r0 + 4 * h + (i >> 2);
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (s16x4 __attribute__((address_space(3)))*)(lds + tile_off<D>(ra, chunk) + byte));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (s16x4 __attribute__((address_space(3)))*)(lds + tile_off<D>(ra + 8, chunk) + byte));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// accumulator registers 8*half .. 8*half+7 of a 32x32 tile as a bf16 B operand
__device__ __forceinline__ bf16x8 acc_to_b(const f32x16& a, int half) {
    bf16x8 r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = (bf16_t)a[8 * half + e];
    return r;
}

// row index inside a 32-row accumulator tile held in register v by a lane of half h
__device__ __forceinline__ int acc_row(int v, int h) { return 8 * (v >> 2) + 4 * h + (v & 3); }

// Heavy-first, then light-last block order for causal masks: the first half of the grid walks the
// query (or key) blocks from the most expensive down, the second half from the cheapest up, so the
// two blocks that share a CU's two slots add up to roughly the same work everywhere.
__device__ __forceinline__ void block_coords(int nblk, int heads, bool causal, bool heavy_is_last_index,
                                            bool paired, int& blk, int& head, int& b) {
    const int per = nblk * heads;             // blocks per batch entry
    const int lin = blockIdx.x % per;
    b = blockIdx.x / per;
    int i = lin / heads;                      // position in the work-sorted order
    head = lin % heads;
    if (causal) {
        // positions 0, 1, 2, ... -> heaviest, lightest, 2nd heaviest, 2nd lightest, ... folded so that
        // the first half of the launch is the heavy half
        // paired: for kernels with two resident blocks per CU; otherwise plain heaviest-first, which
        // lets the hardware hand the light blocks to whichever CU finishes first
        const int half = (nblk + 1) / 2;
        const int rank = !paired ? i : i < half ? i : nblk - 1 - (i - half);      // 0 = heaviest
        blk = heavy_is_last_index ? nblk - 1 - rank : rank;
    } else {
        blk = i;
    }
}

// =====================================================================================
// Forward.  Block = 64 queries = 2 groups of 32 queries x (2 NT) sub-ranges of 32 keys: a step
// covers NT tiles of 64 keys and every wave takes one half of one tile, keeping its own
// online-softmax state; the sub-ranges are merged through LDS at the end.  NT = 1: 4 waves, 64 KB
// (D = 128) of LDS, two blocks per CU.  NT = 2: 8 waves, 128 KB, one block per CU: the heaviest
// causal block then needs half as many steps, and because blocks are dealt out heaviest first
// as CUs become free the tail of the launch stays short.
// =====================================================================================
template <int D, int DR, int NT>
__global__ __launch_bounds__(256 * NT, NT == 1 ? 2 : 1) void attn_fwd_mfma_kernel(AttnArgs a, float scale) {
    constexpr int NW = 4 * NT, NSUB = 2 * NT, KS = D / 16, DT = D / 32;
    constexpr int TILE = 64 * D * 2, STAGE = NT * 2 * TILE;   // per tile: K then V
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int qg = wave / NSUB, sub = wave % NSUB;      // query group; (tile of the step, half of the tile)
    const int tj = sub >> 1, kh = sub & 1;
    const int h = lane >> 5;
    int qblk, head, b;
    block_coords(a.S / 64, a.heads, a.causal != 0, true, NT == 1, qblk, head, b);
    // real head dimension: the tile width (no padding, every guard below folds away), a fixed narrower
    // width (the guards fold to constants), or with DR = 0 whatever the call says
    constexpr bool PAD = DR != D;
    const int dr = DR ? DR : a.d;
    const int H = a.heads * dr, ld = 3 * H;
    const bf16_t* qkv = (const bf16_t*)a.qkv + (size_t)b * a.S * ld + head * dr;
    const bf16_t* kbase = qkv + H;
    const bf16_t* vbase = qkv + 2 * H;
    const int q_wave = qblk * 64 + qg * 32;
    const int q_lane = q_wave + (lane & 31);
    const int klen = a.causal ? a.S : (a.lens ? a.lens[b] : a.S);
    const int kend = a.causal ? qblk * 64 + 64 : klen;     // keys [0, kend) matter to this block
    const int nt = (kend + 63) / 64;                        // tiles
    const int nsteps = (nt + NT - 1) / NT;
    const float c = scale * kLog2e;

    bf16x8 qf[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s)
        qf[s] = load_frag(qkv + (size_t)q_lane * ld, 16 * s + 8 * h, dr);

    f32x16 ot[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) ot[t][v] = 0.f;
    float m = -INFINITY, lsum = 0.f;

    TilePlan<D, NW, PAD> plan;
    plan.init(wave, lane, ld, dr);
    auto request = [&](int step, char* st) {             // the NT tiles of a step (those that exist)
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int k0 = (step * NT + j) * 64;
            if (step * NT + j < nt) {
                plan.issue(kbase + (size_t)k0 * ld, st + j * 2 * TILE, wave);
                plan.issue(vbase + (size_t)k0 * ld, st + j * 2 * TILE + TILE, wave);
            }
        }
    };
    request(0, smem);

    for (int t = 0; t < nsteps; ++t) {
        BP_WAIT_VMCNT(0);
        __syncthreads();
        if (t + 1 < nsteps) request(t + 1, smem + ((t + 1) & 1) * STAGE);
        const int tile = t * NT + tj;
        const int kw = tile * 64 + 32 * kh;             // first key of this wave's sub-range
        if (tile >= nt || (a.causal && kw > q_wave + 31) || kw >= klen) continue;   // nothing unmasked for this wave
        const char* sk = smem + (t & 1) * STAGE + tj * 2 * TILE;
        const char* sv = sk + TILE;

        // S^T (32 keys x 32 queries)
        f32x16 st2;
#pragma unroll
        for (int v = 0; v < 16; ++v) st2[v] = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s)
            if (16 * s < dr)
                st2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(sk, 32 * kh, s, lane), qf[s], st2, 0, 0, 0);
        const bool need_mask = (a.causal && kw + 31 > q_wave) || (kw + 32 > klen);
        float mx = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            float sv_ = st2[v];
            if (need_mask) {
                const int key = kw + acc_row(v, h);
                if ((a.causal && key > q_lane) || key >= klen) sv_ = -INFINITY;
            }
            st2[v] = sv_;
            mx = fmaxf(mx, sv_);
        }
        mx = halves_max(mx) * c;     // c > 0: the maximum commutes with the scaling
        // The reference point m of the running softmax only has to stay within a bounded distance of
        // the true maximum: it moves (and O, l are rescaled) only when some query of the wave sees a
        // score more than 8 binary orders above it, so p <= 2^8 and most tiles skip the rescaling.
        if (__builtin_amdgcn_ballot_w64(mx > m + 8.f) != 0) {
            const float m_new = fmaxf(m, mx);
            const float alpha = m == -INFINITY ? 0.f : fast_exp2(m - m_new);
            m = m_new;
            lsum *= alpha;
#pragma unroll
            for (int t2 = 0; t2 < DT; ++t2)
#pragma unroll
                for (int v = 0; v < 16; ++v) ot[t2][v] *= alpha;
        }
        // a row whose keys are all masked so far keeps m = -inf; avoid inf - inf
        const float m_use = m == -INFINITY ? 0.f : m;
        float ps = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float p = fast_exp2(__builtin_fmaf(st2[v], c, -m_use));
            st2[v] = p;
            ps += p;
        }
        lsum += ps;
        // O^T (D x 32 queries) += V^T P^T over this wave's 32 keys
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            const bf16x8 pb = acc_to_b(st2, s2);
#pragma unroll
            for (int t2 = 0; t2 < DT; ++t2)
                if (32 * t2 < dr)
                    ot[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        frag_cols<D>(sv, 32 * kh + 16 * s2, t2 * 32, lane), pb, ot[t2], 0, 0, 0);
        }
    }

    // merge the key sub-ranges: waves 1 .. NSUB-1 of a query group hand (m, l, O^T) to wave 0 through LDS
    float l = halves_sum(lsum);
    __syncthreads();                                    // all tile reads are over; LDS is free
    constexpr int XO = DT * 16 * 64 + 128;              // [DT*16][64 lanes] + m[64] + l[64]
    float* xo = (float*)smem + (size_t)qg * (NSUB - 1) * XO;
    if (sub != 0) {
        float* mine = xo + (size_t)(sub - 1) * XO;
#pragma unroll
        for (int t2 = 0; t2 < DT; ++t2)
#pragma unroll
            for (int v = 0; v < 16; ++v) mine[(t2 * 16 + v) * 64 + lane] = ot[t2][v];
        mine[DT * 16 * 64 + lane] = m;
        mine[DT * 16 * 64 + 64 + lane] = l;
    }
    __syncthreads();
    if (sub != 0) return;
    float mm = m;                                       // finite: key 0 lies in this wave's sub-range
#pragma unroll
    for (int j = 0; j < NSUB - 1; ++j) mm = fmaxf(mm, xo[(size_t)j * XO + DT * 16 * 64 + lane]);
    const float a0 = fast_exp2(m - mm);
    l *= a0;
#pragma unroll
    for (int t2 = 0; t2 < DT; ++t2)
#pragma unroll
        for (int v = 0; v < 16; ++v) ot[t2][v] *= a0;
#pragma unroll
    for (int j = 0; j < NSUB - 1; ++j) {
        const float* other = xo + (size_t)j * XO;
        const float aj = fast_exp2(other[DT * 16 * 64 + lane] - mm);
        l += other[DT * 16 * 64 + 64 + lane] * aj;
#pragma unroll
        for (int t2 = 0; t2 < DT; ++t2)
#pragma unroll
            for (int v = 0; v < 16; ++v) ot[t2][v] += other[(t2 * 16 + v) * 64 + lane] * aj;
    }
    const float inv = 1.f / l;
    bf16_t* out = (bf16_t*)a.ctx + ((size_t)b * a.S + q_lane) * H + head * dr;
#pragma unroll
    for (int t2 = 0; t2 < DT; ++t2)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint2 pk;
            pk.x = pack_bf16x2(ot[t2][4 * g] * inv, ot[t2][4 * g + 1] * inv);
            pk.y = pack_bf16x2(ot[t2][4 * g + 2] * inv, ot[t2][4 * g + 3] * inv);
            if (t2 * 32 + 8 * g + 4 * h < dr) *reinterpret_cast<uint2*>(out + t2 * 32 + 8 * g + 4 * h) = pk;
        }
    if (h == 0) a.lse[((size_t)b * a.heads + head) * a.S + q_lane] = (mm + log2f(l)) * kLn2;
}

// =====================================================================================
// Backward, part 1: dQ (and delta[q] = sum_d dO[q][d] O[q][d], kept for part 2).  Same decomposition as the forward (lane <-> query, two key halves):
//   S^T = K Q^T, P^T = exp(S^T - lse), dP^T = V dO^T, dS^T = P^T (dP^T - delta),
//   dQ^T (D x 32) += K^T dS^T         (K tile read plainly for S^T and transposed for dQ^T)
// The two halves' partial dQ^T are added through LDS at the end.
// =====================================================================================
template <int D, int DR>
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_mfma_kernel(AttnArgs a, float scale) {
    constexpr int NW = 4, KS = D / 16, DT = D / 32;
    constexpr int TILE = 64 * D * 2, STAGE = 2 * TILE;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int qg = wave >> 1, kh = wave & 1;
    const int h = lane >> 5;
    int qblk, head, b;
    block_coords(a.S / 64, a.heads, a.causal != 0, true, true, qblk, head, b);
    // real head dimension: the tile width (no padding, every guard below folds away), a fixed narrower
    // width (the guards fold to constants), or with DR = 0 whatever the call says
    constexpr bool PAD = DR != D;
    const int dr = DR ? DR : a.d;
    const int H = a.heads * dr, ld = 3 * H;
    const bf16_t* qkv = (const bf16_t*)a.qkv + (size_t)b * a.S * ld + head * dr;
    const bf16_t* kbase = qkv + H;
    const bf16_t* vbase = qkv + 2 * H;
    const int q_wave = qblk * 64 + qg * 32;
    const int q_lane = q_wave + (lane & 31);
    const int klen = a.causal ? a.S : (a.lens ? a.lens[b] : a.S);
    const int kend = a.causal ? qblk * 64 + 64 : klen;
    const int nt = (kend + 63) / 64;
    const float c = scale * kLog2e;

    const bf16_t* dob = (const bf16_t*)a.dctx + ((size_t)b * a.S + q_lane) * H + head * dr;
    bf16x8 qf[KS], dof[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        qf[s] = load_frag(qkv + (size_t)q_lane * ld, 16 * s + 8 * h, dr);
        dof[s] = load_frag(dob, 16 * s + 8 * h, dr);
    }
    const size_t li = ((size_t)b * a.heads + head) * a.S + q_lane;
    const float lse2 = a.lse[li] * kLog2e;
    // delta[q] = sum_d dO[q][d] O[q][d]: each lane holds half of its query's dO row already; the
    // value is also left in a.delta for the dK/dV kernel, which runs after this one
    float delta = 0.f;
    {
        const bf16_t* ob = (const bf16_t*)a.ctx + ((size_t)b * a.S + q_lane) * H + head * dr;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const bf16x8 of = load_frag(ob, 16 * s + 8 * h, dr);
#pragma unroll
            for (int e = 0; e < 8; ++e) delta += (float)of[e] * (float)dof[s][e];
        }
        delta = halves_sum(delta);
        if (kh == 0 && h == 0) a.delta[li] = delta;
    }

    f32x16 dq[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) dq[t][v] = 0.f;

    TilePlan<D, NW, PAD> plan;
    plan.init(wave, lane, ld, dr);
    plan.issue(kbase, smem, wave);
    plan.issue(vbase, smem + TILE, wave);

    for (int t = 0; t < nt; ++t) {
        const int k0 = t * 64;
        BP_WAIT_VMCNT(0);
        __syncthreads();
        if (t + 1 < nt) {
            char* st = smem + ((t + 1) & 1) * STAGE;
            plan.issue(kbase + (size_t)(k0 + 64) * ld, st, wave);
            plan.issue(vbase + (size_t)(k0 + 64) * ld, st + TILE, wave);
        }
        const int kw = k0 + 32 * kh;
        if ((a.causal && kw > q_wave + 31) || kw >= klen) continue;
        const char* sk = smem + (t & 1) * STAGE;
        const char* sv = sk + TILE;
        const bool need_mask = (a.causal && kw + 31 > q_wave) || (kw + 32 > klen);
        f32x16 sacc, dp;
#pragma unroll
        for (int v = 0; v < 16; ++v) { sacc[v] = 0.f; dp[v] = 0.f; }
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            if (16 * s >= dr) continue;
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(sk, 32 * kh, s, lane), qf[s], sacc, 0, 0, 0);
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(sv, 32 * kh, s, lane), dof[s], dp, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            float p = fast_exp2(__builtin_fmaf(sacc[v], c, -lse2));
            if (need_mask) {
                const int key = kw + acc_row(v, h);
                if ((a.causal && key > q_lane) || key >= klen) p = 0.f;
            }
            dp[v] = p * (dp[v] - delta);            // dS^T
        }
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            const bf16x8 db = acc_to_b(dp, s2);
#pragma unroll
            for (int t2 = 0; t2 < DT; ++t2)
                if (32 * t2 < dr)
                    dq[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        frag_cols<D>(sk, 32 * kh + 16 * s2, t2 * 32, lane), db, dq[t2], 0, 0, 0);
        }
    }
    __syncthreads();
    float* xo = (float*)smem + qg * (DT * 16 * 64);
    if (kh == 1) {
#pragma unroll
        for (int t2 = 0; t2 < DT; ++t2)
#pragma unroll
            for (int v = 0; v < 16; ++v) xo[(t2 * 16 + v) * 64 + lane] = dq[t2][v];
    }
    __syncthreads();
    if (kh == 1) return;
    bf16_t* out = (bf16_t*)a.dqkv + ((size_t)b * a.S + q_lane) * ld + head * dr;
#pragma unroll
    for (int t2 = 0; t2 < DT; ++t2)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            float o4[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                o4[e] = (dq[t2][4 * g + e] + xo[(t2 * 16 + 4 * g + e) * 64 + lane]) * scale;
            uint2 pk;
            pk.x = pack_bf16x2(o4[0], o4[1]);
            pk.y = pack_bf16x2(o4[2], o4[3]);
            if (t2 * 32 + 8 * g + 4 * h < dr) *reinterpret_cast<uint2*>(out + t2 * 32 + 8 * g + 4 * h) = pk;
        }
}

// =====================================================================================
// Backward, part 2: dK and dV.  Block = 4 waves = 2 groups of 32 keys x 2 halves of every
// 64-query tile of Q / dO that streams by.
//   S = Q K^T (lane <-> key), P = exp(S - lse[q]), dP = dO V^T, dS = P (dP - delta[q]),
//   dV^T (D x 32 keys) += dO^T P,   dK^T (D x 32 keys) += Q^T dS
// The two query halves' partial sums are added through LDS at the end.
// =====================================================================================
template <int D, int DR>
__global__ __launch_bounds__(256, 2) void attn_bwd_dkv_mfma_kernel(AttnArgs a, float scale) {
    constexpr int NW = 4, KS = D / 16, DT = D / 32;
    constexpr int TILE = 64 * D * 2, STAGE = 2 * TILE + 512;   // Q, dO, then lse[64], delta[64]
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int kg = wave >> 1, qh = wave & 1;
    const int h = lane >> 5;
    int kblk, head, b;
    block_coords(a.S / 64, a.heads, a.causal != 0, false, true, kblk, head, b);   // key block 0 is the heaviest
    // real head dimension: the tile width (no padding, every guard below folds away), a fixed narrower
    // width (the guards fold to constants), or with DR = 0 whatever the call says
    constexpr bool PAD = DR != D;
    const int dr = DR ? DR : a.d;
    const int H = a.heads * dr, ld = 3 * H;
    const bf16_t* qkv = (const bf16_t*)a.qkv + (size_t)b * a.S * ld + head * dr;
    const bf16_t* dobase = (const bf16_t*)a.dctx + (size_t)b * a.S * H + head * dr;
    const int k_wave = kblk * 64 + kg * 32;
    const int k_lane = k_wave + (lane & 31);
    const int klen = a.causal ? a.S : (a.lens ? a.lens[b] : a.S);
    bf16_t* dk_out = (bf16_t*)a.dqkv + ((size_t)b * a.S + k_lane) * ld + H + head * dr;
    bf16_t* dv_out = dk_out + H;
    if (kblk * 64 >= klen) {      // the whole block of keys is padding: no query attends it
        if (qh == 0) {
            const uint2 z = make_uint2(0u, 0u);
#pragma unroll
            for (int t2 = 0; t2 < DT; ++t2)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    if (t2 * 32 + 8 * g + 4 * h >= dr) continue;
                    *reinterpret_cast<uint2*>(dk_out + t2 * 32 + 8 * g + 4 * h) = z;
                    *reinterpret_cast<uint2*>(dv_out + t2 * 32 + 8 * g + 4 * h) = z;
                }
        }
        return;
    }
    const float c = scale * kLog2e;
    const float* lse = a.lse + ((size_t)b * a.heads + head) * a.S;
    const float* dlt = a.delta + ((size_t)b * a.heads + head) * a.S;

    bf16x8 kf[KS], vf[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        kf[s] = load_frag(qkv + H + (size_t)k_lane * ld, 16 * s + 8 * h, dr);
        vf[s] = load_frag(qkv + 2 * H + (size_t)k_lane * ld, 16 * s + 8 * h, dr);
    }
    f32x16 dk[DT], dv[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) { dk[t][v] = 0.f; dv[t][v] = 0.f; }

    const bool pad_in_block = kblk * 64 + 64 > klen;   // some of this block's keys are padding
    const int t0 = a.causal ? kblk : 0;        // first 64-query tile that can see this block's keys
    const int nt = a.S / 64;

    TilePlan<D, NW, PAD> plan_q, plan_do;
    plan_q.init(wave, lane, ld, dr);
    plan_do.init(wave, lane, H, dr);
    auto load_stage = [&](int t, char* st) {
        const int q0 = t * 64;
        plan_q.issue(qkv + (size_t)q0 * ld, st, wave);
        plan_do.issue(dobase + (size_t)q0 * H, st + TILE, wave);
        // the tile's 64 log-sum-exp values and 64 deltas travel the same way (4 bytes per lane): a load
        // into registers followed by an LDS store would make these waves wait for the tile loads
        // issued just before it, i.e. for the whole memory latency, in every step
        if (wave == 0)
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(lse + q0 + lane),
                                             (void __attribute__((address_space(3)))*)(st + 2 * TILE), 4, 0, 0);
        else if (wave == 1)
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(dlt + q0 + lane),
                                             (void __attribute__((address_space(3)))*)(st + 2 * TILE + 256), 4, 0, 0);
    };
    load_stage(t0, smem + (t0 & 1) * STAGE);

    for (int t = t0; t < nt; ++t) {
        const int q0 = t * 64;
        BP_WAIT_VMCNT(0);
        __syncthreads();
        if (t + 1 < nt) load_stage(t + 1, smem + ((t + 1) & 1) * STAGE);
        const int qw = q0 + 32 * qh;                     // first query of this wave's half
        if (a.causal && qw + 31 < k_wave) continue;      // no query of this half reaches this wave's keys
        const char* sq = smem + (t & 1) * STAGE;
        const char* sdo = sq + TILE;
        const float* s_lse = (const float*)(sq + 2 * TILE) + 32 * qh;
        const float* s_dlt = (const float*)(sq + 2 * TILE) + 64 + 32 * qh;
        const bool need_mask = a.causal && qw < k_wave + 31;
        f32x16 sacc, dp;
#pragma unroll
        for (int v = 0; v < 16; ++v) { sacc[v] = 0.f; dp[v] = 0.f; }
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            if (16 * s >= dr) continue;
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(sq, 32 * qh, s, lane), kf[s], sacc, 0, 0, 0);
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<D>(sdo, 32 * qh, s, lane), vf[s], dp, 0, 0, 0);
        }
        // masked scores become -inf before the exponential (p = 0, dS = 0); both conditions are
        // wave-uniform branches, taken only on the diagonal tile and in a block with padded keys
        if (need_mask) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (k_lane > qw + acc_row(v, h)) sacc[v] = -INFINITY;
        }
        if (pad_in_block && k_lane >= klen) {
#pragma unroll
            for (int v = 0; v < 16; ++v) sacc[v] = -INFINITY;
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int qi = acc_row(v, h);
            const float p = fast_exp2(__builtin_fmaf(sacc[v], c, -s_lse[qi] * kLog2e));
            sacc[v] = p;                                 // P
            dp[v] = p * (dp[v] - s_dlt[qi]);             // dS
        }
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            const bf16x8 pb = acc_to_b(sacc, s2);
            const bf16x8 db = acc_to_b(dp, s2);
#pragma unroll
            for (int t2 = 0; t2 < DT; ++t2) {
                if (32 * t2 >= dr) continue;
                dv[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    frag_cols<D>(sdo, 32 * qh + 16 * s2, t2 * 32, lane), pb, dv[t2], 0, 0, 0);
                dk[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    frag_cols<D>(sq, 32 * qh + 16 * s2, t2 * 32, lane), db, dk[t2], 0, 0, 0);
            }
        }
    }
    __syncthreads();
    float* xo = (float*)smem + kg * (2 * DT * 16 * 64);
    if (qh == 1) {
#pragma unroll
        for (int t2 = 0; t2 < DT; ++t2)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                xo[(t2 * 16 + v) * 64 + lane] = dk[t2][v];
                xo[((DT + t2) * 16 + v) * 64 + lane] = dv[t2][v];
            }
    }
    __syncthreads();
    if (qh == 1) return;
#pragma unroll
    for (int t2 = 0; t2 < DT; ++t2)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            float k4[4], v4[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                k4[e] = (dk[t2][4 * g + e] + xo[(t2 * 16 + 4 * g + e) * 64 + lane]) * scale;
                v4[e] = dv[t2][4 * g + e] + xo[((DT + t2) * 16 + 4 * g + e) * 64 + lane];
            }
            if (t2 * 32 + 8 * g + 4 * h >= dr) continue;
            uint2 pk;
            pk.x = pack_bf16x2(k4[0], k4[1]);
            pk.y = pack_bf16x2(k4[2], k4[3]);
            *reinterpret_cast<uint2*>(dk_out + t2 * 32 + 8 * g + 4 * h) = pk;
            pk.x = pack_bf16x2(v4[0], v4[1]);
            pk.y = pack_bf16x2(v4[2], v4[3]);
            *reinterpret_cast<uint2*>(dv_out + t2 * 32 + 8 * g + 4 * h) = pk;
        }
}

// ---- host side
bool attn_mfma_supported(const AttnArgs& a) {
    auto al16 = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
    if (a.d % 8 || a.d < 8 || a.d > 128) return false;      // tile width 64 or 128, narrower heads are padded
    if (a.S % 64) return false;
    return al16(a.qkv) && al16(a.ctx) && (!a.dctx || al16(a.dctx)) && (!a.dqkv || al16(a.dqkv));
}

template <typename K>
static hipError_t set_smem(K kern, size_t smem) {
    if (smem <= 64 * 1024) return hipSuccess;
    return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
}

// Tiles of 64 keys per forward step.  Two (8 waves, one block per CU) halve the step count of the
// heaviest causal block, which is what bounds a launch with only a couple of blocks per CU; with
// many blocks per CU the 4-wave form with two co-resident blocks is faster.
static int tiles_per_step(const AttnArgs& a) {
    static std::atomic<int> n_cu_cached{0};
    int n_cu = n_cu_cached.load(std::memory_order_relaxed);
    if (!n_cu) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0)
            n_cu = 256;
        n_cu_cached.store(n_cu, std::memory_order_relaxed);
    }
    const long blocks = (long)(a.S / 64) * a.heads * a.B;
    return (a.S >= 512 && blocks <= 2L * n_cu) ? 2 : 1;
}

template <int D, int DR, int NT>
static hipError_t launch_fwd_nt(const AttnArgs& a, hipStream_t s) {
    const float scale = 1.f / sqrtf((float)a.d);
    const dim3 grid((a.S / 64) * a.heads * a.B), block(256 * NT);
    const size_t stages = (size_t)2 * NT * 2 * 64 * D * 2;
    const size_t merge = (size_t)2 * (2 * NT - 1) * ((D / 32) * 16 * 64 + 128) * sizeof(float);
    const size_t smem = stages > merge ? stages : merge;
    static std::atomic<bool> set{false};   // several host threads may launch at once
    if (!set.load(std::memory_order_acquire)) {
        hipError_t e = set_smem(attn_fwd_mfma_kernel<D, DR, NT>, smem);
        if (e != hipSuccess) return e;
        set.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((attn_fwd_mfma_kernel<D, DR, NT>), grid, block, smem, s, a, scale);
    return hipGetLastError();
}
template <int D, int DR>
static hipError_t launch_fwd_t(const AttnArgs& a, hipStream_t s) {
    return tiles_per_step(a) == 2 ? launch_fwd_nt<D, DR, 2>(a, s) : launch_fwd_nt<D, DR, 1>(a, s);
}

hipError_t launch_attn_fwd_mfma(const AttnArgs& a, hipStream_t s) {
    if (a.d == 128) return launch_fwd_t<128, 128>(a, s);
    if (a.d == 64) return launch_fwd_t<64, 64>(a, s);
    // the head widths of the paper's own models (Table 3) get kernels with the width built in
    if (a.d == 96) return launch_fwd_t<128, 96>(a, s);
    if (a.d == 40) return launch_fwd_t<64, 40>(a, s);
    return a.d > 64 ? launch_fwd_t<128, 0>(a, s) : launch_fwd_t<64, 0>(a, s);
}

template <int D, int DR>
static hipError_t launch_bwd_t(const AttnArgs& a, hipStream_t s) {
    const float scale = 1.f / sqrtf((float)a.d);
    const dim3 grid((a.S / 64) * a.heads * a.B), block(256);
    const size_t smem = 2 * 2 * 64 * D * 2, smem2 = 2 * (2 * 64 * D * 2 + 512);
    static std::atomic<bool> set{false};   // several host threads may launch at once
    if (!set.load(std::memory_order_acquire)) {
        hipError_t e = set_smem(attn_bwd_dq_mfma_kernel<D, DR>, smem);
        if (e == hipSuccess) e = set_smem(attn_bwd_dkv_mfma_kernel<D, DR>, smem2);
        if (e != hipSuccess) return e;
        set.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<D, DR>), grid, block, smem, s, a, scale);
    hipLaunchKernelGGL((attn_bwd_dkv_mfma_kernel<D, DR>), grid, block, smem2, s, a, scale);
    return hipGetLastError();
}

hipError_t launch_attn_bwd_mfma(const AttnArgs& a, hipStream_t s) {
    if (a.d == 128) return launch_bwd_t<128, 128>(a, s);
    if (a.d == 64) return launch_bwd_t<64, 64>(a, s);
    if (a.d == 96) return launch_bwd_t<128, 96>(a, s);
    if (a.d == 40) return launch_bwd_t<64, 40>(a, s);
    return a.d > 64 ? launch_bwd_t<128, 0>(a, s) : launch_bwd_t<64, 0>(a, s);
}

}  // namespace bp
