// Shape-generic kernels: a tiled GEMM with fp32 accumulation and a row-at-a-time attention
// forward/backward.  They serve the fp32 storage path (tiny, latency-bound shapes) and any bf16
// shape the MFMA kernels do not cover; correctness first, no tuning.
#include "bp_kernels.h"
#include "bp_device.h"

namespace bp {

// ------------------------------------------------------------------ GEMM 64x64x16, 4x4 per thread
template <typename T>
__global__ __launch_bounds__(256) void gemm_generic_kernel(GemmArgs g) {
    __shared__ float As[16][65];
    __shared__ float Bs[16][65];
    const T* A = (const T*)g.A;
    const T* B = (const T*)g.B;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < g.K; k0 += 16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = threadIdx.x + i * 256;
            int m, k;
            if (g.a_t) { k = e >> 6; m = e & 63; } else { m = e >> 4; k = e & 15; }
            const int gm = m0 + m, gk = k0 + k;
            float v = 0.f;
            if (gm < g.M && gk < g.K)
                v = to_float<T>(g.a_t ? A[(size_t)gk * g.lda + gm] : A[(size_t)gm * g.lda + gk]);
            As[k][m] = v;
            int n;
            if (g.b_t) { n = e >> 4; k = e & 15; } else { k = e >> 6; n = e & 63; }
            const int gn = n0 + n;
            const int gk2 = k0 + k;
            v = 0.f;
            if (gn < g.N && gk2 < g.K)
                v = to_float<T>(g.b_t ? B[(size_t)gn * g.ldb + gk2] : B[(size_t)gk2 * g.ldb + gn]);
            Bs[k][n] = v;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= g.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= g.N) continue;
            float v = acc[i][j];
            const size_t o = (size_t)m * g.ldc + n;
            if (g.accumulate) {
                float* c = (float*)g.C + o;
                *c = g.accumulate == 2 ? v : *c + v;
            } else {
                if (g.bias) v += g.bias[n];
                if (g.residual) v += to_float<T>(((const T*)g.residual)[o]);
                ((T*)g.C)[o] = from_float<T>(v);
            }
        }
    }
}

hipError_t launch_gemm_generic(int dtype, const GemmArgs& g, hipStream_t s) {
    if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipErrorInvalidValue;
    dim3 grid((g.N + 63) / 64, (g.M + 63) / 64), block(256);
    if (dtype == BF16)
        hipLaunchKernelGGL((gemm_generic_kernel<bf16_t>), grid, block, 0, s, g);
    else
        hipLaunchKernelGGL((gemm_generic_kernel<float>), grid, block, 0, s, g);
    return hipGetLastError();
}

// ------------------------------------------------------------------ attention, one query row per block
__device__ __forceinline__ float block_reduce(float v, float* red, bool is_max) {
    v = is_max ? wave_max(v) : wave_sum(v);
    const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float r = red[0];
    for (int i = 1; i < nw; ++i) r = is_max ? fmaxf(r, red[i]) : r + red[i];
    return r;
}

template <typename T>
__global__ __launch_bounds__(128) void attn_fwd_generic_kernel(AttnArgs a, float scale) {
    extern __shared__ float smem[];
    float* sc = smem;             // [S]
    float* qs = sc + a.S;         // [d]
    float* red = qs + a.d;        // [4]
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int H = a.heads * a.d, ld = 3 * H;
    const T* qkv = (const T*)a.qkv;
    const T* qrow = qkv + ((size_t)(b * a.S + i)) * ld + h * a.d;
    const T* kbase = qkv + ((size_t)b * a.S) * ld + H + h * a.d;
    const T* vbase = kbase + H;
    const int kend = a.causal ? i + 1 : (a.lens ? a.lens[b] : a.S);
    for (int c = threadIdx.x; c < a.d; c += blockDim.x) qs[c] = to_float<T>(qrow[c]);
    __syncthreads();
    float mx = -INFINITY;
    for (int j = threadIdx.x; j < kend; j += blockDim.x) {
        const T* kr = kbase + (size_t)j * ld;
        float dot = 0.f;
        for (int c = 0; c < a.d; ++c) dot += qs[c] * to_float<T>(kr[c]);
        dot *= scale;
        sc[j] = dot;
        mx = fmaxf(mx, dot);
    }
    mx = block_reduce(mx, red, true);
    float sum = 0.f;
    for (int j = threadIdx.x; j < kend; j += blockDim.x) {
        const float e = __expf(sc[j] - mx);
        sc[j] = e;
        sum += e;
    }
    sum = block_reduce(sum, red, false);
    const float inv = 1.f / sum;
    T* out = (T*)a.ctx + ((size_t)(b * a.S + i)) * H + h * a.d;
    for (int c = threadIdx.x; c < a.d; c += blockDim.x) {
        float acc = 0.f;
        for (int j = 0; j < kend; ++j) acc += sc[j] * to_float<T>(vbase[(size_t)j * ld + c]);
        out[c] = from_float<T>(acc * inv);
    }
    if (threadIdx.x == 0) a.lse[((size_t)b * a.heads + h) * a.S + i] = mx + __logf(sum);
}

// dq and delta, one query row per block
template <typename T>
__global__ __launch_bounds__(128) void attn_bwd_dq_generic_kernel(AttnArgs a, float scale) {
    extern __shared__ float smem[];
    float* ds = smem;             // [S]
    float* qs = ds + a.S;         // [d]
    float* dos = qs + a.d;        // [d]
    float* red = dos + a.d;       // [4]
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int H = a.heads * a.d, ld = 3 * H;
    const T* qkv = (const T*)a.qkv;
    const size_t tok = (size_t)(b * a.S + i);
    const T* qrow = qkv + tok * ld + h * a.d;
    const T* kbase = qkv + ((size_t)b * a.S) * ld + H + h * a.d;
    const T* vbase = kbase + H;
    const T* orow = (const T*)a.ctx + tok * H + h * a.d;
    const T* dorow = (const T*)a.dctx + tok * H + h * a.d;
    const int kend = a.causal ? i + 1 : (a.lens ? a.lens[b] : a.S);
    float part = 0.f;
    for (int c = threadIdx.x; c < a.d; c += blockDim.x) {
        qs[c] = to_float<T>(qrow[c]);
        const float dv = to_float<T>(dorow[c]);
        dos[c] = dv;
        part += dv * to_float<T>(orow[c]);
    }
    const float delta = block_reduce(part, red, false);
    const size_t li = ((size_t)b * a.heads + h) * a.S + i;
    const float lse = a.lse[li];
    if (threadIdx.x == 0) a.delta[li] = delta;
    for (int j = threadIdx.x; j < kend; j += blockDim.x) {
        const T* kr = kbase + (size_t)j * ld;
        const T* vr = vbase + (size_t)j * ld;
        float s = 0.f, dp = 0.f;
        for (int c = 0; c < a.d; ++c) {
            s += qs[c] * to_float<T>(kr[c]);
            dp += dos[c] * to_float<T>(vr[c]);
        }
        const float p = __expf(s * scale - lse);
        ds[j] = p * (dp - delta);
    }
    __syncthreads();
    T* dq = (T*)a.dqkv + tok * ld + h * a.d;
    for (int c = threadIdx.x; c < a.d; c += blockDim.x) {
        float acc = 0.f;
        for (int j = 0; j < kend; ++j) acc += ds[j] * to_float<T>(kbase[(size_t)j * ld + c]);
        dq[c] = from_float<T>(acc * scale);
    }
}

// dk and dv, one key row per block (needs delta from the dq kernel)
template <typename T>
__global__ __launch_bounds__(128) void attn_bwd_dkv_generic_kernel(AttnArgs a, float scale) {
    extern __shared__ float smem[];
    float* ps = smem;             // [S]
    float* dss = ps + a.S;        // [S]
    float* ks = dss + a.S;        // [d]
    float* vs = ks + a.d;         // [d]
    const int j = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int H = a.heads * a.d, ld = 3 * H;
    const T* qkv = (const T*)a.qkv;
    const size_t tok = (size_t)(b * a.S + j);
    const T* qbase = qkv + ((size_t)b * a.S) * ld + h * a.d;
    const T* krow = qkv + tok * ld + H + h * a.d;
    const T* vrow = krow + H;
    const T* dobase = (const T*)a.dctx + ((size_t)b * a.S) * H + h * a.d;
    T* dk = (T*)a.dqkv + tok * ld + H + h * a.d;
    T* dv = dk + H;
    const int klen = a.causal ? a.S : (a.lens ? a.lens[b] : a.S);
    if (j >= klen) {   // masked key: no query attends it
        for (int c = threadIdx.x; c < a.d; c += blockDim.x) {
            dk[c] = from_float<T>(0.f);
            dv[c] = from_float<T>(0.f);
        }
        return;
    }
    const int i0 = a.causal ? j : 0;
    for (int c = threadIdx.x; c < a.d; c += blockDim.x) {
        ks[c] = to_float<T>(krow[c]);
        vs[c] = to_float<T>(vrow[c]);
    }
    __syncthreads();
    const float* lse = a.lse + ((size_t)b * a.heads + h) * a.S;
    const float* delta = a.delta + ((size_t)b * a.heads + h) * a.S;
    for (int i = i0 + threadIdx.x; i < a.S; i += blockDim.x) {
        const T* qr = qbase + (size_t)i * ld;
        const T* dor = dobase + (size_t)i * H;
        float s = 0.f, dp = 0.f;
        for (int c = 0; c < a.d; ++c) {
            s += to_float<T>(qr[c]) * ks[c];
            dp += to_float<T>(dor[c]) * vs[c];
        }
        const float p = __expf(s * scale - lse[i]);
        ps[i] = p;
        dss[i] = p * (dp - delta[i]);
    }
    __syncthreads();
    for (int c = threadIdx.x; c < a.d; c += blockDim.x) {
        float av = 0.f, ak = 0.f;
        for (int i = i0; i < a.S; ++i) {
            av += ps[i] * to_float<T>(dobase[(size_t)i * H + c]);
            ak += dss[i] * to_float<T>(qbase[(size_t)i * ld + c]);
        }
        dv[c] = from_float<T>(av);
        dk[c] = from_float<T>(ak * scale);
    }
}

hipError_t launch_attn_fwd_generic(int dtype, const AttnArgs& a, hipStream_t s) {
    const float scale = 1.f / sqrtf((float)a.d);
    dim3 grid(a.S, a.heads, a.B), block(128);
    const size_t sm = (size_t)(a.S + a.d + 8) * sizeof(float);
    if (sm > 60000) return hipErrorInvalidValue;
    if (dtype == BF16)
        hipLaunchKernelGGL((attn_fwd_generic_kernel<bf16_t>), grid, block, sm, s, a, scale);
    else
        hipLaunchKernelGGL((attn_fwd_generic_kernel<float>), grid, block, sm, s, a, scale);
    return hipGetLastError();
}

hipError_t launch_attn_bwd_generic(int dtype, const AttnArgs& a, hipStream_t s) {
    const float scale = 1.f / sqrtf((float)a.d);
    dim3 grid(a.S, a.heads, a.B), block(128);
    const size_t sm1 = (size_t)(a.S + 2 * a.d + 8) * sizeof(float);
    const size_t sm2 = (size_t)(2 * a.S + 2 * a.d) * sizeof(float);
    if (sm1 > 60000 || sm2 > 60000) return hipErrorInvalidValue;
    if (dtype == BF16) {
        hipLaunchKernelGGL((attn_bwd_dq_generic_kernel<bf16_t>), grid, block, sm1, s, a, scale);
        hipLaunchKernelGGL((attn_bwd_dkv_generic_kernel<bf16_t>), grid, block, sm2, s, a, scale);
    } else {
        hipLaunchKernelGGL((attn_bwd_dq_generic_kernel<float>), grid, block, sm1, s, a, scale);
        hipLaunchKernelGGL((attn_bwd_dkv_generic_kernel<float>), grid, block, sm2, s, a, scale);
    }
    return hipGetLastError();
}

}  // namespace bp
