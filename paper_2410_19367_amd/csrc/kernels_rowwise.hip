// Bandwidth-bound kernels of the stage: LayerNorm forward/backward (+ residual-gradient add),
// bias+GELU forward/backward, column reductions for bias and LayerNorm parameter gradients,
// the synthetic loss, and small utilities.  All are one pass over their data with 16-byte
// accesses per lane; statistics and math are fp32 whatever the storage type.
#include "bp_kernels.h"
#include "bp_device.h"

namespace bp {

// ------------------------------------------------------------------ LayerNorm forward
// One 64-lane wave per row; the row lives in registers (NP passes of 64 lanes x 8 columns).
template <typename T, int NP>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const T* __restrict__ x,
                                                     const float* __restrict__ gamma,
                                                     const float* __restrict__ beta,
                                                     T* __restrict__ out, float* __restrict__ mean,
                                                     float* __restrict__ rstd, T* __restrict__ xcopy,
                                                     int rows, int H, float eps) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const T* xr = x + (size_t)row * H;
    float v[NP][8];
    float s = 0.f;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int col = (p * 64 + lane) * 8;
        if (col < H) {
            load8(xr + col, v[p]);
            if (xcopy) store8(xcopy + (size_t)row * H + col, v[p]);
#pragma unroll
            for (int i = 0; i < 8; ++i) s += v[p][i];
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[p][i] = 0.f;
        }
    }
    const float mu = wave_sum(s) / (float)H;
    float q = 0.f;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int col = (p * 64 + lane) * 8;
        if (col < H) {
#pragma unroll
            for (int i = 0; i < 8; ++i) { const float d = v[p][i] - mu; q += d * d; }
        }
    }
    const float rs = rsqrtf(wave_sum(q) / (float)H + eps);
    if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int col = (p * 64 + lane) * 8;
        if (col < H) {
            float g[8], b[8], o[8];
            load8(gamma + col, g);
            load8(beta + col, b);
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = (v[p][i] - mu) * rs * g[i] + b[i];
            store8(out + (size_t)row * H + col, o);
        }
    }
}

// ------------------------------------------------------------------ LayerNorm backward (rows)
// dx = res + rstd * (dxhat - mean(dxhat) - xhat * mean(dxhat * xhat)), dxhat = dout * gamma.
template <typename T, int NP>
__global__ __launch_bounds__(256) void ln_bwd_rows_kernel(const T* __restrict__ dout,
                                                          const T* __restrict__ x,
                                                          const float* __restrict__ mean,
                                                          const float* __restrict__ rstd,
                                                          const float* __restrict__ gamma,
                                                          const T* __restrict__ res,
                                                          T* __restrict__ dx, int rows, int H) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const size_t base = (size_t)row * H;
    const float mu = mean[row], rs = rstd[row];
    float xh[NP][8], dh[NP][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int col = (p * 64 + lane) * 8;
        if (col < H) {
            float g[8];
            load8(x + base + col, xh[p]);
            load8(dout + base + col, dh[p]);
            load8(gamma + col, g);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                xh[p][i] = (xh[p][i] - mu) * rs;
                dh[p][i] *= g[i];
                s1 += dh[p][i];
                s2 += dh[p][i] * xh[p][i];
            }
        }
    }
    s1 = wave_sum(s1) / (float)H;
    s2 = wave_sum(s2) / (float)H;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int col = (p * 64 + lane) * 8;
        if (col < H) {
            float r[8], o[8];
            if (res) load8(res + base + col, r);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                o[i] = rs * (dh[p][i] - s1 - xh[p][i] * s2);
                if (res) o[i] += r[i];
            }
            store8(dx + base + col, o);
        }
    }
}

// ------------------------------------------------------------------ column reductions
// Several reductions over [T, N_j] tensors run as one batch (blockIdx.x walks the column blocks of
// all jobs, blockIdx.y the row chunks).  Block = 4 waves
// covering 512 columns x kColsumRows rows; wave w takes rows w, w+4, ... and requests all of
// them before consuming the first.  Partials are combined across the waves in LDS and written
// per row chunk; a second kernel folds the chunks in a fixed order, so the result does not
// depend on scheduling.
template <typename T>
__global__ __launch_bounds__(256) void colsum_partial_kernel(ColsumBatch batch, int rows) {
    __shared__ float red[2][4][576];
    // blockIdx.x runs over the column blocks of all jobs one after the other
    int ji = 0;
    while (ji + 1 < batch.n && (int)blockIdx.x >= batch.first_block[ji + 1]) ++ji;
    const ColsumJob job = batch.jobs[ji];
    const int N = job.N;
    const int cb = blockIdx.x - batch.first_block[ji];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int col = cb * 512 + lane * 8;
    const T* A = (const T*)job.A;
    const T* X = (const T*)job.X;
    const bool with_x = X != nullptr;
    const int r0 = blockIdx.y * kColsumRows;
    const int r1 = min(r0 + kColsumRows, rows);
    float sa[8] = {0, 0, 0, 0, 0, 0, 0, 0}, sx[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (col < N) {
        // a wave's 8 rows in two groups of 4: all loads of a group are in flight together, and the
        // register footprint stays small enough for every block of the launch to be resident
        constexpr int RPW = kColsumRows / 4, GRP = 4;
        float mu[RPW], rs[RPW];                          // row statistics, requested before the rows
        if (with_x) {
#pragma unroll
            for (int j = 0; j < RPW; ++j) {
                const int r = min(r0 + w + 4 * j, rows - 1);
                mu[j] = job.mean[r];
                rs[j] = job.rstd[r];
            }
        }
#pragma unroll
        for (int j0 = 0; j0 < RPW; j0 += GRP) {
            float a[GRP][8], xv[GRP][8];
#pragma unroll
            for (int j = 0; j < GRP; ++j) {
                const int r = r0 + w + 4 * (j0 + j);
                if (r < r1) {
                    load8(A + (size_t)r * N + col, a[j]);
                    if (with_x) load8(X + (size_t)r * N + col, xv[j]);
                }
            }
#pragma unroll
            for (int j = 0; j < GRP; ++j) {
                const int r = r0 + w + 4 * (j0 + j);
                if (r < r1) {
                    if (with_x) {
#pragma unroll
                        for (int i = 0; i < 8; ++i) sx[i] += a[j][i] * (xv[j][i] - mu[j0 + j]) * rs[j0 + j];
                    }
#pragma unroll
                    for (int i = 0; i < 8; ++i) sa[i] += a[j][i];
                }
            }
        }
    }
    // lane-major with a pitch of 9 floats: conflict-free for the writes and for the reads below
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        red[0][w][lane * 9 + i] = sa[i];
        red[1][w][lane * 9 + i] = sx[i];
    }
    __syncthreads();
    const int nout = with_x ? 2 : 1;
    for (int e = threadIdx.x; e < 512 * nout; e += 256) {
        const int o = e / 512, c = e % 512;
        const int gc = cb * 512 + c;
        if (gc < N) {
            const int a = (c >> 3) * 9 + (c & 7);
            const float v = (red[o][0][a] + red[o][1][a]) + (red[o][2][a] + red[o][3][a]);
            job.part[((size_t)blockIdx.y * nout + o) * N + gc] = v;
        }
    }
}

// out_k[c] += (or =, for a batch marked overwrite) sum over chunks of part[chunk][k][c].  Block = 64 columns x 4 chunk slices.
__global__ __launch_bounds__(256) void colsum_final_kernel(ColsumBatch batch, int chunks) {
    __shared__ float red[4][64];
    const ColsumJob job = batch.jobs[blockIdx.y];
    const int N = job.N;
    if (blockIdx.x * 64 >= N || !job.part) return;
    const int nout = job.out_ax ? 2 : 1;
    const int cl = threadIdx.x & 63, slice = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + cl;
    for (int o = 0; o < nout; ++o) {
        float s = 0.f;
        if (c < N) {
            // 16 loads in flight per thread (the additions keep their order): with 4 the kernel
            // spends its time waiting for one memory latency after the other
#pragma unroll 16
            for (int k = slice; k < chunks; k += 4) s += job.part[((size_t)k * nout + o) * N + c];
        }
        red[slice][cl] = s;
        __syncthreads();
        if (slice == 0 && c < N) {
            float* out = o == 0 ? job.out_a : job.out_ax;
            const float v = (red[0][cl] + red[1][cl]) + (red[2][cl] + red[3][cl]);
            out[c] = batch.overwrite ? v : out[c] + v;
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------ bias + GELU
template <typename T>
__global__ __launch_bounds__(256) void gelu_fwd_kernel(const T* __restrict__ u,
                                                       const float* __restrict__ bias,
                                                       T* __restrict__ g, int rows, int F) {
    const int vec_per_row = F / 8;
    const size_t total = (size_t)rows * vec_per_row;
    for (size_t v = (size_t)blockIdx.x * 256 + threadIdx.x; v < total; v += (size_t)gridDim.x * 256) {
        const int col = (int)(v % vec_per_row) * 8;
        float a[8], b[8], o[8];
        load8(u + v * 8, a);
        load8(bias + col, b);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float x = a[i] + b[i];
            o[i] = gelu_value(x);
        }
        store8(g + v * 8, o);
    }
}

// du = dg * gelu'(u + b); partial column sums of du per row chunk (same scheme as colsum).
template <typename T>
__global__ __launch_bounds__(256) void gelu_bwd_kernel(const T* dg,   // may alias du
                                                       const T* __restrict__ u,
                                                       const float* __restrict__ bias,
                                                       T* du, float* __restrict__ part,
                                                       int rows, int F) {
    __shared__ float red[4][576];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int col = blockIdx.x * 512 + lane * 8;
    const int r0 = blockIdx.y * kColsumRows;
    const int r1 = min(r0 + kColsumRows, rows);
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (col < F) {
        float b[8];
        load8(bias + col, b);
        constexpr int RPW = kColsumRows / 4, GRP = 4;
#pragma unroll
        for (int j0 = 0; j0 < RPW; j0 += GRP) {
            float a[GRP][8], d[GRP][8];
#pragma unroll
            for (int j = 0; j < GRP; ++j) {
                const int r = r0 + w + 4 * (j0 + j);
                if (r < r1) {
                    load8(u + (size_t)r * F + col, a[j]);
                    load8(dg + (size_t)r * F + col, d[j]);
                }
            }
#pragma unroll
            for (int j = 0; j < GRP; ++j) {
                const int r = r0 + w + 4 * (j0 + j);
                if (r < r1) {
                    float o[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const float x = a[j][i] + b[i];
                        o[i] = d[j][i] * gelu_slope(x);
                        acc[i] += o[i];
                    }
                    store8(du + (size_t)r * F + col, o);
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) red[w][lane * 9 + i] = acc[i];
    __syncthreads();
    for (int c = threadIdx.x; c < 512; c += 256) {
        const int gc = blockIdx.x * 512 + c;
        const int a = (c >> 3) * 9 + (c & 7);
        if (gc < F)
            part[(size_t)blockIdx.y * F + gc] = (red[0][a] + red[1][a]) + (red[2][a] + red[3][a]);
    }
}

// ------------------------------------------------------------------ loss
template <typename T>
__global__ __launch_bounds__(256) void loss_partial_kernel(const T* __restrict__ z,
                                                           const T* __restrict__ y, float scale,
                                                           T* __restrict__ grad,
                                                           float* __restrict__ part, size_t n) {
    __shared__ float red[4];
    float s = 0.f;
    const size_t nv = n / 8;
    for (size_t v = (size_t)blockIdx.x * 256 + threadIdx.x; v < nv; v += (size_t)gridDim.x * 256) {
        float a[8], b[8], o[8];
        load8(z + v * 8, a);
        load8(y + v * 8, b);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float d = a[i] - b[i];
            s += d * d;
            o[i] = d * scale;
        }
        store8(grad + v * 8, o);
    }
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) part[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ __launch_bounds__(256) void loss_final_kernel(const float* __restrict__ part, int nparts,
                                                         float scale, float* __restrict__ out) {
    __shared__ float red[4];
    float s = 0.f;
    for (int i = threadIdx.x; i < nparts; i += 256) s += part[i];
    s = wave_sum(s);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) out[0] = 0.5f * scale * ((red[0] + red[1]) + (red[2] + red[3]));
}

// ------------------------------------------------------------------ utilities
__global__ __launch_bounds__(256) void fill_f32_kernel(float* p, size_t n, float v) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
        p[i] = v;
}
__global__ __launch_bounds__(256) void add_f32_kernel(float* dst, const float* src, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
        dst[i] += src[i];
}
template <typename T>
__global__ __launch_bounds__(256) void cast_from_f32_kernel(const float* src, T* dst, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
        dst[i] = from_float<T>(src[i]);
}

// dst[c][r] = src[r][c] through a padded 32x32 LDS tile
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T* __restrict__ src, T* __restrict__ dst,
                                                        int rows, int cols) {
    __shared__ T tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;      // 32 x 8
    const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    for (int i = ty; i < 32; i += 8)
        if (r0 + i < rows && c0 + tx < cols) tile[i][tx] = src[(size_t)(r0 + i) * cols + c0 + tx];
    __syncthreads();
    for (int i = ty; i < 32; i += 8)
        if (c0 + i < cols && r0 + tx < rows) dst[(size_t)(c0 + i) * rows + r0 + tx] = tile[tx][i];
}

// ------------------------------------------------------------------ launchers
static inline int grid_for(size_t work_items, int per_block, int cap = 256 * 16) {
    size_t b = (work_items + per_block - 1) / per_block;
    if (b < 1) b = 1;
    return (int)(b > (size_t)cap ? cap : b);
}

template <typename T>
static hipError_t ln_fwd_dispatch(int T_, int H, const T* x, const float* gamma, const float* beta,
                                  float eps, T* out, float* mean, float* rstd, T* xcopy,
                                  hipStream_t s) {
    const int np = (H + 511) / 512;
    dim3 grid((T_ + 3) / 4), block(256);
#define BP_LN_CASE(NPV)                                                                        \
    if (np <= NPV) {                                                                           \
        hipLaunchKernelGGL((ln_fwd_kernel<T, NPV>), grid, block, 0, s, x, gamma, beta, out,    \
                           mean, rstd, xcopy, T_, H, eps);                                     \
        return hipGetLastError();                                                              \
    }
    BP_LN_CASE(1) BP_LN_CASE(2) BP_LN_CASE(4) BP_LN_CASE(6) BP_LN_CASE(8) BP_LN_CASE(10)
    BP_LN_CASE(16)
#undef BP_LN_CASE
    return hipErrorInvalidValue;
}

template <typename T>
static hipError_t ln_bwd_dispatch(int T_, int H, const T* dout, const T* x, const float* mean,
                                  const float* rstd, const float* gamma, const T* res, T* dx,
                                  hipStream_t s) {
    const int np = (H + 511) / 512;
    dim3 grid((T_ + 3) / 4), block(256);
#define BP_LN_CASE(NPV)                                                                        \
    if (np <= NPV) {                                                                           \
        hipLaunchKernelGGL((ln_bwd_rows_kernel<T, NPV>), grid, block, 0, s, dout, x, mean,     \
                           rstd, gamma, res, dx, T_, H);                                       \
        return hipGetLastError();                                                              \
    }
    BP_LN_CASE(1) BP_LN_CASE(2) BP_LN_CASE(4) BP_LN_CASE(6) BP_LN_CASE(8) BP_LN_CASE(10)
    BP_LN_CASE(16)
#undef BP_LN_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_ln_fwd(int dtype, int T, int H, const void* x, const float* gamma,
                         const float* beta, float eps, void* out, float* mean, float* rstd,
                         void* xcopy, hipStream_t s) {
    if (H % 8 || H > 8192 || T <= 0) return hipErrorInvalidValue;
    if (dtype == BF16)
        return ln_fwd_dispatch<bf16_t>(T, H, (const bf16_t*)x, gamma, beta, eps, (bf16_t*)out, mean,
                                       rstd, (bf16_t*)xcopy, s);
    return ln_fwd_dispatch<float>(T, H, (const float*)x, gamma, beta, eps, (float*)out, mean, rstd,
                                  (float*)xcopy, s);
}

hipError_t launch_ln_bwd_rows(int dtype, int T, int H, const void* dout, const void* x,
                              const float* mean, const float* rstd, const float* gamma,
                              const void* res, void* dx, hipStream_t s) {
    if (H % 8 || H > 8192 || T <= 0) return hipErrorInvalidValue;
    if (dtype == BF16)
        return ln_bwd_dispatch<bf16_t>(T, H, (const bf16_t*)dout, (const bf16_t*)x, mean, rstd, gamma,
                                       (const bf16_t*)res, (bf16_t*)dx, s);
    return ln_bwd_dispatch<float>(T, H, (const float*)dout, (const float*)x, mean, rstd, gamma,
                                  (const float*)res, (float*)dx, s);
}

hipError_t launch_colsum_batch(int dtype, int T, const ColsumBatch& batch, hipStream_t s) {
    if (T <= 0 || batch.n <= 0 || batch.n > kMaxColsumJobs) return hipErrorInvalidValue;
    const int chunks = (int)colsum_chunks(T);
    int max_n = 0;
    bool any_partial = false;
    for (int j = 0; j < batch.n; ++j) {
        if (batch.jobs[j].N % 8) return hipErrorInvalidValue;
        max_n = max_n > batch.jobs[j].N ? max_n : batch.jobs[j].N;
        any_partial |= batch.jobs[j].A != nullptr;
    }
    if (any_partial) {
        ColsumBatch b2 = batch;
        int nb = 0;
        for (int j = 0; j < batch.n; ++j) {
            b2.first_block[j] = nb;
            if (batch.jobs[j].A) nb += (batch.jobs[j].N + 511) / 512;
        }
        b2.first_block[batch.n] = nb;
        dim3 grid(nb, chunks), block(256);
        if (dtype == BF16) hipLaunchKernelGGL((colsum_partial_kernel<bf16_t>), grid, block, 0, s, b2, T);
        else hipLaunchKernelGGL((colsum_partial_kernel<float>), grid, block, 0, s, b2, T);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(colsum_final_kernel, dim3((max_n + 63) / 64, batch.n), dim3(256), 0, s, batch, chunks);
    return hipGetLastError();
}

hipError_t launch_colsum(int dtype, int T, int N, const void* A, const void* X, const float* mean,
                         const float* rstd, float* out_a, float* out_ax, float* ws, hipStream_t s) {
    ColsumBatch b;
    b.n = 1;
    b.jobs[0] = ColsumJob{A, X, mean, rstd, N, out_a, X ? out_ax : nullptr, ws};
    return launch_colsum_batch(dtype, T, b, s);
}

hipError_t launch_gelu_fwd(int dtype, int T, int F, const void* u, const float* bias, void* g,
                           hipStream_t s) {
    if (F % 8 || T <= 0) return hipErrorInvalidValue;
    const int grid = grid_for((size_t)T * F / 8, 256, 256 * 32);
    if (dtype == BF16)
        hipLaunchKernelGGL((gelu_fwd_kernel<bf16_t>), dim3(grid), dim3(256), 0, s, (const bf16_t*)u,
                           bias, (bf16_t*)g, T, F);
    else
        hipLaunchKernelGGL((gelu_fwd_kernel<float>), dim3(grid), dim3(256), 0, s, (const float*)u,
                           bias, (float*)g, T, F);
    return hipGetLastError();
}

hipError_t launch_gelu_bwd(int dtype, int T, int F, const void* dg, const void* u,
                           const float* bias, void* du, float* dbias, float* ws, hipStream_t s) {
    // dbias == nullptr: leave the per-chunk partials in ws for a later batched final reduction
    if (F % 8 || T <= 0) return hipErrorInvalidValue;
    const int chunks = (int)colsum_chunks(T);
    dim3 grid((F + 511) / 512, chunks), block(256);
    if (dtype == BF16)
        hipLaunchKernelGGL((gelu_bwd_kernel<bf16_t>), grid, block, 0, s, (const bf16_t*)dg,
                           (const bf16_t*)u, bias, (bf16_t*)du, ws, T, F);
    else
        hipLaunchKernelGGL((gelu_bwd_kernel<float>), grid, block, 0, s, (const float*)dg,
                           (const float*)u, bias, (float*)du, ws, T, F);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !dbias) return e;
    ColsumBatch b;
    b.n = 1;
    b.jobs[0] = ColsumJob{nullptr, nullptr, nullptr, nullptr, F, dbias, nullptr, ws};
    hipLaunchKernelGGL(colsum_final_kernel, dim3((F + 63) / 64, 1), block, 0, s, b, chunks);
    return hipGetLastError();
}

hipError_t launch_loss(int dtype, size_t n, const void* z, const void* target, float scale,
                       void* grad, float* loss_out, float* ws, hipStream_t s) {
    if (n % 8) return hipErrorInvalidValue;
    const int grid = grid_for(n / 8, 256, 1024);
    if (dtype == BF16)
        hipLaunchKernelGGL((loss_partial_kernel<bf16_t>), dim3(grid), dim3(256), 0, s,
                           (const bf16_t*)z, (const bf16_t*)target, scale, (bf16_t*)grad, ws, n);
    else
        hipLaunchKernelGGL((loss_partial_kernel<float>), dim3(grid), dim3(256), 0, s,
                           (const float*)z, (const float*)target, scale, (float*)grad, ws, n);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(loss_final_kernel, dim3(1), dim3(256), 0, s, ws, grid, scale, loss_out);
    return hipGetLastError();
}

hipError_t launch_fill_f32(float* p, size_t n, float v, hipStream_t s) {
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(fill_f32_kernel, dim3(grid_for(n, 256 * 4)), dim3(256), 0, s, p, n, v);
    return hipGetLastError();
}
hipError_t launch_add_f32(float* dst, const float* src, size_t n, hipStream_t s) {
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(add_f32_kernel, dim3(grid_for(n, 256 * 4)), dim3(256), 0, s, dst, src, n);
    return hipGetLastError();
}
hipError_t launch_transpose(int dtype, int rows, int cols, const void* src, void* dst, hipStream_t s) {
    if (rows <= 0 || cols <= 0) return hipErrorInvalidValue;
    dim3 grid((cols + 31) / 32, (rows + 31) / 32), block(256);
    if (dtype == BF16)
        hipLaunchKernelGGL((transpose_kernel<bf16_t>), grid, block, 0, s, (const bf16_t*)src, (bf16_t*)dst, rows, cols);
    else
        hipLaunchKernelGGL((transpose_kernel<float>), grid, block, 0, s, (const float*)src, (float*)dst, rows, cols);
    return hipGetLastError();
}

hipError_t launch_cast_from_f32(int dtype, const float* src, void* dst, size_t n, hipStream_t s) {
    if (n == 0) return hipSuccess;
    const int grid = grid_for(n, 256 * 4);
    if (dtype == BF16)
        hipLaunchKernelGGL((cast_from_f32_kernel<bf16_t>), dim3(grid), dim3(256), 0, s, src,
                           (bf16_t*)dst, n);
    else
        hipLaunchKernelGGL((cast_from_f32_kernel<float>), dim3(grid), dim3(256), 0, s, src,
                           (float*)dst, n);
    return hipGetLastError();
}

}  // namespace bp
