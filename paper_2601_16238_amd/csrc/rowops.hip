// Row-wise neighbours of attention for gfx950: RMSNorm forward, LayerNorm forward and
// backward, rotary forward.  All are bound by HBM traffic: every activation element is read
// once and written once, a whole row lives in the registers of one work-group between the
// reduction and the normalisation, 16-byte accesses throughout.
#include "../../include/attn.h"
#include "../../include/rowops.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rowops {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;          // threads that share one row
constexpr int kWaves = kThreads / 64;
constexpr int kMaxCols = 16384;        // 8 vectors of 8 elements per thread
constexpr int kBwdTeams = 512;         // rows above which the LayerNorm backward pairs its row teams

__device__ __forceinline__ bf16x8 load8(const __bf16 *p)
{
    return __builtin_bit_cast(bf16x8, *(const u32x4 *)p);
}
__device__ __forceinline__ void store8(__bf16 *p, const float (&v)[8])
{
    typedef float f32x8 __attribute__((ext_vector_type(8)));
    f32x8 f = {v[0], v[1], v[2], v[3], v[4], v[5], v[6], v[7]};
    *(u32x4 *)p = __builtin_bit_cast(u32x4, __builtin_convertvector(f, bf16x8));
}
__device__ __forceinline__ void load8f(const float *p, float (&v)[8])
{
    const f32x4 a = *(const f32x4 *)p, b = *(const f32x4 *)(p + 4);
    v[0] = a[0]; v[1] = a[1]; v[2] = a[2]; v[3] = a[3];
    v[4] = b[0]; v[5] = b[1]; v[6] = b[2]; v[7] = b[3];
}

// Sum of N values per thread over the work-group; every thread gets the result.  `red` is
// LDS scratch of kWaves * N floats; the trailing barrier makes it reusable at once.
template <int N>
__device__ __forceinline__ void block_sum(float (&v)[N], float *red)
{
#pragma unroll
    for (int n = 0; n < N; ++n)
#pragma unroll
        for (int s = 32; s >= 1; s >>= 1) v[n] += __shfl_xor(v[n], s);
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0)
#pragma unroll
        for (int n = 0; n < N; ++n) red[w * N + n] = v[n];
    __syncthreads();
#pragma unroll
    for (int n = 0; n < N; ++n) {
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < kWaves; ++i) t += red[i * N + n];
        v[n] = t;
    }
    __syncthreads();
}

// Thread t owns vectors t, t + 256, ... (V of them) of 8 consecutive columns each.
template <int V>
__device__ __forceinline__ void load_row(const __bf16 *row, int cols, float (&x)[V][8])
{
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int c = (threadIdx.x + v * kThreads) * 8;
        if (c < cols) {
            const bf16x8 b = load8(row + c);
#pragma unroll
            for (int e = 0; e < 8; ++e) x[v][e] = (float)b[e];
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) x[v][e] = 0.f;
        }
    }
}

// Raw 16-byte vectors of a row, fetched one row ahead by the kernels that walk several rows.
// With four or more vectors per thread the loads are unconditional (vectors past the row's end
// re-read its first one; unpack_row zeroes them) and the widened values are pinned by an empty
// asm, so that the widening stays ahead of the next fetch into the same raw registers and the
// compiler can count the loads it waits for: -1 % at 8192 columns, -6 % at 16384.  Narrower
// rows, whose three or four resident work-groups per unit already cover the latency, are
// 5-8 % faster in the plain form.
template <int V>
__device__ __forceinline__ void fetch_row(const __bf16 *row, int cols, u32x4 (&raw)[V], int t)
{
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int c = (t + v * kThreads) * 8;
        if constexpr (V >= 4) raw[v] = *(const u32x4 *)(row + (c < cols ? c : 0));
        else if (c < cols) raw[v] = *(const u32x4 *)(row + c);
    }
}
template <int V>
__device__ __forceinline__ void unpack_row(const u32x4 (&raw)[V], int cols, float (&x)[V][8], int t)
{
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int c = (t + v * kThreads) * 8;
        const bf16x8 b = __builtin_bit_cast(bf16x8, raw[v]);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            x[v][e] = c < cols ? (float)b[e] : 0.f;
            if constexpr (V >= 4) asm volatile("" : "+v"(x[v][e]));
        }
    }
}

// The forward kernels run a fixed number of work-groups (see fwd_groups);
// each walks rows group, group + G, ... with its slice of the parameters in registers (loaded
// once instead of once per row) and fetches its next row while it works on the current one.
template <int V>
__global__ void __launch_bounds__(kThreads)
rmsnorm_fwd_kernel(const __bf16 *x, const float *w, __bf16 *y, int64_t rows, int cols, int64_t xs,
                   int64_t ys, float eps)
{
    __shared__ float red[kWaves];
    float wv[V][8];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int c = (threadIdx.x + v * kThreads) * 8;
        if (c < cols) load8f(w + c, wv[v]);
    }
    u32x4 nx[V] = {};
    if ((int64_t)blockIdx.x < rows) fetch_row<V>(x + blockIdx.x * xs, cols, nx, threadIdx.x);
    for (int64_t i = blockIdx.x; i < rows; i += gridDim.x) {
        float xv[V][8];
        unpack_row<V>(nx, cols, xv, threadIdx.x);
        if (i + gridDim.x < rows) fetch_row<V>(x + (i + gridDim.x) * xs, cols, nx, threadIdx.x);
        float ss[1] = {0.f};
#pragma unroll
        for (int v = 0; v < V; ++v)
#pragma unroll
            for (int e = 0; e < 8; ++e) ss[0] += xv[v][e] * xv[v][e];
        block_sum<1>(ss, red);
        const float r = 1.0f / sqrtf(ss[0] / (float)cols + eps);
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const int c = (threadIdx.x + v * kThreads) * 8;
            if (c < cols) {
                float o[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = xv[v][e] * r * wv[v][e];
                store8(y + i * ys + c, o);
            }
        }
    }
}

template <int V>
__global__ void __launch_bounds__(kThreads)
layernorm_fwd_kernel(const __bf16 *x, const float *w, const float *b, __bf16 *y, float *mean,
                     float *rstd, int64_t rows, int cols, int64_t xs, int64_t ys, float eps)
{
    __shared__ float red[kWaves];
    float wv[V][8], bv[V][8];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int c = (threadIdx.x + v * kThreads) * 8;
        if (c < cols) {
            load8f(w + c, wv[v]);
            load8f(b + c, bv[v]);
        }
    }
    u32x4 nx[V] = {};
    if ((int64_t)blockIdx.x < rows) fetch_row<V>(x + blockIdx.x * xs, cols, nx, threadIdx.x);
    for (int64_t i = blockIdx.x; i < rows; i += gridDim.x) {
        float xv[V][8];
        unpack_row<V>(nx, cols, xv, threadIdx.x);
        if (i + gridDim.x < rows) fetch_row<V>(x + (i + gridDim.x) * xs, cols, nx, threadIdx.x);
        float s[1] = {0.f};
#pragma unroll
        for (int v = 0; v < V; ++v)
#pragma unroll
            for (int e = 0; e < 8; ++e) s[0] += xv[v][e];
        block_sum<1>(s, red);
        const float mu = s[0] / (float)cols;
        // second pass over the registers: the variance of the centred values
        float q[1] = {0.f};
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const int c = (threadIdx.x + v * kThreads) * 8;
            if (c < cols)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    xv[v][e] -= mu;
                    q[0] += xv[v][e] * xv[v][e];
                }
        }
        block_sum<1>(q, red);
        const float r = 1.0f / sqrtf(q[0] / (float)cols + eps);
        if (threadIdx.x == 0) {
            mean[i] = mu;
            rstd[i] = r;
        }
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const int c = (threadIdx.x + v * kThreads) * 8;
            if (c < cols) {
                float o[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = xv[v][e] * r * wv[v][e] + bv[v][e];
                store8(y + i * ys + c, o);
            }
        }
    }
}

// Backward.  A work-group is T teams of kThreads threads; each team takes one row at a time
// (round j of the work-group covers rows (j * G + group) * T + team) and computes its dx.  The
// column sums of dw and db stay in registers across a team's rows; at the end the teams add
// theirs together through LDS, in team order, and the work-group writes one partial row:
// part[g][0][cols] = dw, part[g][1][cols] = db.  More teams per work-group mean fewer partial
// rows to write here and to read in the column kernel, at the same number of waves per unit.
template <int V, int T>
__global__ void __launch_bounds__(kThreads * T)
layernorm_bwd_rows_kernel(const __bf16 *dy, const __bf16 *x, const float *w, const float *mean,
                          const float *rstd, __bf16 *dx, float *part, int64_t rows, int cols,
                          int64_t dys, int64_t xs, int64_t dxs)
{
    __shared__ float red[T * kWaves * 2];
    __shared__ float comb[T > 1 ? 16 * kThreads : 1];
    const int t = threadIdx.x % kThreads, team = threadIdx.x / kThreads;
    float wv[V][8], dwp[V][8], dbp[V][8];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int c = (t + v * kThreads) * 8;
        if (c < cols) load8f(w + c, wv[v]);
#pragma unroll
        for (int e = 0; e < 8; ++e) { dwp[v][e] = 0.f; dbp[v][e] = 0.f; }
    }
    // A team walks its rows one after the other, so the next row is fetched (as raw 16-byte
    // vectors) before the current one is worked on: its HBM latency then overlaps the
    // arithmetic, the two reductions and the stores of the current row.
    u32x4 nx[V] = {}, ng[V] = {};
    float nmu = 0.f, nr = 0.f;
    // (vectors past the row's end re-read its first one, so that every thread issues the same
    // loads and the wait for them can be counted; unpack_row zeroes those vectors)
    auto fetch = [&](int64_t i) __attribute__((always_inline)) {
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const int c = (t + v * kThreads) * 8;
            nx[v] = *(const u32x4 *)(x + i * xs + (c < cols ? c : 0));
            ng[v] = *(const u32x4 *)(dy + i * dys + (c < cols ? c : 0));
        }
        nmu = mean[i];
        nr = rstd[i];
    };
    const int64_t step = (int64_t)gridDim.x * T;
    if ((int64_t)blockIdx.x * T + team < rows) fetch((int64_t)blockIdx.x * T + team);
    // `base` is the same for every thread of the work-group, so all of them reach the barriers
    // of every round; a team whose row lies past the end contributes zeros and stores nothing.
    for (int64_t base = (int64_t)blockIdx.x * T; base < rows; base += step) {
        const int64_t i = base + team;
        const bool live = i < rows;
        float xv[V][8], gv[V][8];
        float s[2] = {0.f, 0.f};  // sum g, sum g*xhat with g = dy*w
        // (the fetch stands outside the `live` branch so that its registers are not merged
        // with another path at the branch's end, which would make the wave wait for them there)
        unpack_row<V>(nx, cols, xv, t);
        unpack_row<V>(ng, cols, gv, t);
        const float mu = nmu, r = nr;
        // the row is unpacked here, before the raw registers are loaded again
#pragma unroll
        for (int v = 0; v < V; ++v)
#pragma unroll
            for (int e = 0; e < 8; ++e) asm volatile("" : "+v"(xv[v][e]), "+v"(gv[v][e]));
        if (i + step < rows) fetch(i + step);
        if (live) {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const int c = (t + v * kThreads) * 8;
                if (c < cols)
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        xv[v][e] = (xv[v][e] - mu) * r;  // xhat
                        dwp[v][e] += gv[v][e] * xv[v][e];
                        dbp[v][e] += gv[v][e];
                        gv[v][e] *= wv[v][e];            // g
                        s[0] += gv[v][e];
                        s[1] += gv[v][e] * xv[v][e];
                    }
            }
        }
        // sums over the team
#pragma unroll
        for (int n = 0; n < 2; ++n)
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) s[n] += __shfl_xor(s[n], m);
        if ((threadIdx.x & 63) == 0) {
            red[(threadIdx.x >> 6) * 2 + 0] = s[0];
            red[(threadIdx.x >> 6) * 2 + 1] = s[1];
        }
        __syncthreads();
        s[0] = s[1] = 0.f;
#pragma unroll
        for (int k = 0; k < kWaves; ++k) {
            s[0] += red[(team * kWaves + k) * 2 + 0];
            s[1] += red[(team * kWaves + k) * 2 + 1];
        }
        __syncthreads();
        if (live) {
            const float mg = s[0] / (float)cols, mgx = s[1] / (float)cols;
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const int c = (t + v * kThreads) * 8;
                if (c < cols) {
                    float o[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] = r * (gv[v][e] - mg - xv[v][e] * mgx);
                    store8(dx + i * dxs + c, o);
                }
            }
        }
    }
    // teams 1 .. T-1 hand their column sums to team 0, one vector slot at a time
    if (T > 1) {
#pragma unroll
        for (int v = 0; v < V; ++v)
            for (int k = 1; k < T; ++k) {
                if (team == k)
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        comb[e * kThreads + t] = dwp[v][e];
                        comb[(8 + e) * kThreads + t] = dbp[v][e];
                    }
                __syncthreads();
                if (team == 0)
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        dwp[v][e] += comb[e * kThreads + t];
                        dbp[v][e] += comb[(8 + e) * kThreads + t];
                    }
                __syncthreads();
            }
    }
    if (team != 0) return;
    float *pw = part + (int64_t)blockIdx.x * 2 * cols, *pb = pw + cols;
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int c = (t + v * kThreads) * 8;
        if (c < cols)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                f32x4 a, b;
#pragma unroll
                for (int e = 0; e < 4; ++e) { a[e] = dwp[v][4 * h + e]; b[e] = dbp[v][4 * h + e]; }
                *(f32x4 *)(pw + c + 4 * h) = a;
                *(f32x4 *)(pb + c + 4 * h) = b;
            }
    }
}

// Column reduction of the partial sums.  The rows of `part` are [group][dw | db][cols], i.e.
// 2 * cols floats per group.  A work-group owns W consecutive floats of that row (W / 4 lanes
// x 4) and splits the groups over 1024 / W slices, so that enough loads are in flight to cover
// HBM latency; the slices are then summed through LDS in a fixed order (deterministic).
template <int W>
__global__ void __launch_bounds__(256)
layernorm_bwd_cols_kernel(const float *part, float *dw, float *db, int groups, int cols)
{
    constexpr int kLanes = W / 4, kSlices = 256 / kLanes;
    __shared__ f32x4 red[kSlices][kLanes];
    const int q = threadIdx.x % kLanes, slice = threadIdx.x / kLanes;
    const int c = blockIdx.x * W + q * 4;  // position within the 2 * cols floats of a group
    const bool in_range = c < 2 * cols;    // the last work-group may be ragged
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    if (in_range)
        for (int g = slice; g < groups; g += kSlices)
            acc += *(const f32x4 *)(part + (int64_t)g * 2 * cols + c);
    red[slice][q] = acc;
    __syncthreads();
    if (slice == 0 && in_range) {
        f32x4 t = red[0][q];
#pragma unroll
        for (int i = 1; i < kSlices; ++i) t += red[i][q];
        *(f32x4 *)((c < cols ? dw : db - cols) + c) = t;
    }
}

// Rotary: one thread per 8 pairs (d..d+7, d+hd..d+hd+7) of one (b, h, s) row.
__global__ void __launch_bounds__(256)
rotary_fwd_kernel(const __bf16 *x, const float *cosv, const float *sinv, __bf16 *y, int H, int S,
                  int D, int64_t rows, int64_t xsb, int64_t xsh, int64_t xss, int64_t ysb,
                  int64_t ysh, int64_t yss)
{
    const int hd = D / 2, tpr = hd / 8;  // threads per row
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t row = t / tpr;
    if (row >= rows) return;
    const int d = (int)(t % tpr) * 8;
    const int s = (int)(row % S), h = (int)((row / S) % H);
    const int64_t b = row / ((int64_t)S * H);
    const __bf16 *xr = x + b * xsb + h * xsh + (int64_t)s * xss;
    __bf16 *yr = y + b * ysb + h * ysh + (int64_t)s * yss;
    const bf16x8 lo = load8(xr + d), hi = load8(xr + d + hd);
    float c[8], sn[8], o1[8], o2[8];
    load8f(cosv + (int64_t)s * hd + d, c);
    load8f(sinv + (int64_t)s * hd + d, sn);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float a = (float)lo[e], bb = (float)hi[e];
        // (written out as fused multiply-adds: the rotation fused into the attention
        // forward's Q load uses the same two expressions and gives the same bits)
        o1[e] = __builtin_fmaf(a, c[e], -(bb * sn[e]));
        o2[e] = __builtin_fmaf(bb, c[e], a * sn[e]);
    }
    store8(yr + d, o1);
    store8(yr + d + hd, o2);
}

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int check_rows(int64_t rows, int32_t cols, std::initializer_list<int64_t> strides)
{
    if (rows < 1 || rows > 0x7fffffffLL || cols < 8 || cols > kMaxCols || cols % 8) return ATTN_ERR_SHAPE;
    for (int64_t s : strides)
        if (s < cols || s % 8) return ATTN_ERR_STRIDE;
    return ATTN_OK;
}

// LayerNorm backward: row teams per work-group, and work-groups.  The launch is one round of
// resident work-groups.  Up to 4 vectors per thread a work-group is two teams once there are
// rows for more than 512 teams: the same waves per unit in half the work-groups, so half the
// partial rows to write and to sum.  Teams per unit (more cost partial rows, fewer leave
// latency uncovered), measured on (16384, 1024), (8192, 4096), (4096, 8192), (2048, 16384):
// V = 1: 4 (33.7 us; 44.8 with 2, 39.1 with 3), V = 2: 2 (38.3 us; 44.7 with 3; 41.3 as
// single-team work-groups), V = 4: 2, all its registers allow (40.3 us; 44.4 as single-team
// work-groups in two rounds), V = 8: 1 (50.3 us; 63.4 with 2).
int bwd_teams(int64_t rows, int V) { return rows > kBwdTeams && V <= 4 ? 2 : 1; }
int bwd_groups(int64_t rows, int V)
{
    const int T = bwd_teams(rows, V);
    const int teams_per_cu = V == 1 ? 4 : V == 8 ? 1 : 2;
    const int64_t g = (rows + T - 1) / T, cap = 256 * teams_per_cu / T;
    return (int)(g < cap ? g : cap);
}
// Work-groups of the forward kernels: as many as are resident at once on the 256 compute units
// for the kernel's register use at V vectors per thread (8 waves per SIMD at most), so that
// the launch is a single round.  Measured on (4096, 8192): LayerNorm 28.1 us with one
// work-group per row, 24.8 us with 1024 groups, 23.2 us with 768 (three fit a unit).
int fwd_groups(int64_t rows, int V, bool layernorm)
{
    const int per_cu = V == 1 ? 8 : V == 2 ? 4 : V == 4 ? (layernorm ? 3 : 4) : 2;
    const int64_t g = 256 * per_cu;
    return (int)(rows < g ? rows : g);
}

// vectors per thread: 1, 2, 4 or 8
int vectors_for(int cols)
{
    const int v = (cols / 8 + kThreads - 1) / kThreads;
    return v <= 1 ? 1 : v <= 2 ? 2 : v <= 4 ? 4 : 8;
}

#define ROWOPS_DISPATCH(V, CALL)            \
    switch (V) {                            \
        case 1: { constexpr int kV = 1; CALL; } break; \
        case 2: { constexpr int kV = 2; CALL; } break; \
        case 4: { constexpr int kV = 4; CALL; } break; \
        default: { constexpr int kV = 8; CALL; } break; \
    }

}  // namespace rowops

using namespace rowops;

extern "C" {

int rowops_rmsnorm_fwd(const void *x, const float *w, void *y, int64_t rows, int32_t cols,
                       int64_t x_row_stride, int64_t y_row_stride, float eps, void *hip_stream)
{
    if (!x || !w || !y) return ATTN_ERR_NULL;
    const int rc = check_rows(rows, cols, {x_row_stride, y_row_stride});
    if (rc != ATTN_OK) return rc;
    if (!aligned(x, 16) || !aligned(w, 16) || !aligned(y, 16)) return ATTN_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    ROWOPS_DISPATCH(vectors_for(cols),
        hipLaunchKernelGGL((rmsnorm_fwd_kernel<kV>), dim3(fwd_groups(rows, kV, false)), dim3(kThreads), 0, st,
                           static_cast<const __bf16 *>(x), w, static_cast<__bf16 *>(y), rows, cols,
                           x_row_stride, y_row_stride, eps));
    return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}

int rowops_layernorm_fwd(const void *x, const float *w, const float *b, void *y, float *mean,
                         float *rstd, int64_t rows, int32_t cols, int64_t x_row_stride,
                         int64_t y_row_stride, float eps, void *hip_stream)
{
    if (!x || !w || !b || !y || !mean || !rstd) return ATTN_ERR_NULL;
    const int rc = check_rows(rows, cols, {x_row_stride, y_row_stride});
    if (rc != ATTN_OK) return rc;
    if (!aligned(x, 16) || !aligned(w, 16) || !aligned(b, 16) || !aligned(y, 16) ||
        !aligned(mean, 4) || !aligned(rstd, 4))
        return ATTN_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    ROWOPS_DISPATCH(vectors_for(cols),
        hipLaunchKernelGGL((layernorm_fwd_kernel<kV>), dim3(fwd_groups(rows, kV, true)), dim3(kThreads), 0, st,
                           static_cast<const __bf16 *>(x), w, b, static_cast<__bf16 *>(y), mean,
                           rstd, rows, cols, x_row_stride, y_row_stride, eps));
    return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}

size_t rowops_layernorm_bwd_workspace_bytes(int64_t rows, int32_t cols)
{
    if (check_rows(rows, cols, {}) != ATTN_OK) return 0;
    const size_t bytes = (size_t)bwd_groups(rows, vectors_for(cols)) * 2 * cols * sizeof(float);
    return (bytes + 255) / 256 * 256;
}

int rowops_layernorm_bwd(const void *dy, const void *x, const float *w, const float *mean,
                         const float *rstd, void *dx, float *dw, float *db,
                         void *workspace, size_t workspace_bytes, int64_t rows, int32_t cols,
                         int64_t dy_row_stride, int64_t x_row_stride, int64_t dx_row_stride,
                         void *hip_stream)
{
    if (!dy || !x || !w || !mean || !rstd || !dx || !dw || !db) return ATTN_ERR_NULL;
    const int rc = check_rows(rows, cols, {dy_row_stride, x_row_stride, dx_row_stride});
    if (rc != ATTN_OK) return rc;
    if (!aligned(dy, 16) || !aligned(x, 16) || !aligned(w, 16) || !aligned(dx, 16) ||
        !aligned(dw, 16) || !aligned(db, 16) || !aligned(mean, 4) || !aligned(rstd, 4))
        return ATTN_ERR_ALIGN;
    if (!workspace || !aligned(workspace, 256) ||
        workspace_bytes < rowops_layernorm_bwd_workspace_bytes(rows, cols))
        return ATTN_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int V = vectors_for(cols), groups = bwd_groups(rows, V);
    float *part = static_cast<float *>(workspace);
#define ROWOPS_LN_BWD(T)                                                                          \
    hipLaunchKernelGGL((layernorm_bwd_rows_kernel<kV, T>), dim3(groups), dim3(kThreads * T), 0,   \
                       st, static_cast<const __bf16 *>(dy), static_cast<const __bf16 *>(x), w,    \
                       mean, rstd, static_cast<__bf16 *>(dx), part, rows, cols, dy_row_stride,    \
                       x_row_stride, dx_row_stride)
    if (bwd_teams(rows, V) == 2) {
        switch (V) {
            case 1: { constexpr int kV = 1; ROWOPS_LN_BWD(2); } break;
            case 2: { constexpr int kV = 2; ROWOPS_LN_BWD(2); } break;
            default: { constexpr int kV = 4; ROWOPS_LN_BWD(2); } break;
        }
    } else {
        ROWOPS_DISPATCH(V, ROWOPS_LN_BWD(1));
    }
#undef ROWOPS_LN_BWD
    if (hipGetLastError() != hipSuccess) return ATTN_ERR_LAUNCH;
    // 2 * cols floats per group, W per work-group: 16 for rows below 4096 columns, so that the
    // launch still has a few hundred work-groups ((16384, 1024): 38.0 -> 34.5 us; 8 is slower)
#define ROWOPS_LN_COLS(W)                                                                         \
    hipLaunchKernelGGL((layernorm_bwd_cols_kernel<W>), dim3((2 * cols + W - 1) / W), dim3(256), 0, \
                       st, part, dw, db, groups, cols)
    if (cols < 4096) ROWOPS_LN_COLS(16);
    else ROWOPS_LN_COLS(32);
#undef ROWOPS_LN_COLS
    return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}

int rowops_rotary_fwd(const void *x, const float *cos_table, const float *sin_table, void *y,
                      int32_t B, int32_t H, int32_t S, int32_t D,
                      int64_t x_stride_b, int64_t x_stride_h, int64_t x_stride_s,
                      int64_t y_stride_b, int64_t y_stride_h, int64_t y_stride_s,
                      void *hip_stream)
{
    if (!x || !cos_table || !sin_table || !y) return ATTN_ERR_NULL;
    if (B < 1 || H < 1 || S < 1 || D < 16 || D > 512 || D % 16) return ATTN_ERR_SHAPE;
    const int64_t rows = (int64_t)B * H * S;
    if (rows * (D / 16) > 0x7fffffffLL * 256) return ATTN_ERR_SHAPE;
    for (int64_t s : {x_stride_b, x_stride_h, x_stride_s, y_stride_b, y_stride_h, y_stride_s})
        if (s < 1 || s % 8) return ATTN_ERR_STRIDE;
    if (x_stride_s < D || y_stride_s < D) return ATTN_ERR_STRIDE;
    if (!aligned(x, 16) || !aligned(y, 16) || !aligned(cos_table, 16) || !aligned(sin_table, 16))
        return ATTN_ERR_ALIGN;
    const int64_t threads = rows * (D / 16);
    hipLaunchKernelGGL(rotary_fwd_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<const __bf16 *>(x),
                       cos_table, sin_table, static_cast<__bf16 *>(y), H, S, D, rows, x_stride_b,
                       x_stride_h, x_stride_s, y_stride_b, y_stride_h, y_stride_s);
    return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}

}  // extern "C"
