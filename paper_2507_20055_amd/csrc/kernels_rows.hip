// Row-streaming kernels of the back-substitution: ReLU relaxation parameters, the sign-split
// ReLU step (+ bias fold), concretisation, margin rows, verdict.  All HBM-bound: one wavefront
// streams one coefficient row with 16-byte loads, per-input parameters sit in LDS, the per-row
// constant is accumulated in fp64 and reduced with wavefront shuffles.
#include <algorithm>

#include "common.h"

namespace dpc {

namespace {

constexpr int kThreads = 256;          // 4 wavefronts of 64
constexpr int kWaves = kThreads / 64;
constexpr int kMaxRowsPerWave = 8;
constexpr int kChunk = 2048;           // columns of per-input parameters resident in LDS at a time

typedef float vfloat4 __attribute__((ext_vector_type(4)));

// Streaming (non-temporal) 16-byte accesses: coefficient rows are touched once per kernel.
__device__ __forceinline__ float4 nt_load4(const float4* p)
{
    const vfloat4 v = __builtin_nontemporal_load(reinterpret_cast<const vfloat4*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void nt_store4(float4* p, float a, float b, float c, float d)
{
    vfloat4 v = {a, b, c, d};
    __builtin_nontemporal_store(v, reinterpret_cast<vfloat4*>(p));
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// DeepPoly ReLU transformer (Appendix C: relu, relu_n, compute_upper), one thread per neuron.
__global__ __launch_bounds__(kThreads) void relax_params_kernel(
    const float* __restrict__ l, const float* __restrict__ u, float* __restrict__ lambda,
    float* __restrict__ mu, float* __restrict__ nu, float* __restrict__ rl, float* __restrict__ ru,
    int64_t count)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= count) return;
    const float lv = l[i], uv = u[i];
    lambda[i] = (lv + uv >= 0.0f) ? 1.0f : 0.0f;
    float m, v;
    if (lv >= 0.0f) { m = 1.0f; v = 0.0f; }
    else if (uv <= 0.0f) { m = 0.0f; v = 0.0f; }
    else {
        const float d = uv - lv;
        m = uv / d;
        v = -(uv * lv) / d;
    }
    mu[i] = m;
    nu[i] = v;
    rl[i] = lv >= 0.0f ? lv : 0.0f;
    ru[i] = uv >= 0.0f ? uv : 0.0f;
}

// Parameters of the sign-split ReLU step for columns [c0, c0 + cw) of input b into LDS: multiplier for C >= 0, multiplier
// for C < 0, and the constant picked up per unit of C >= 0 / C < 0 (nu on the side that uses U, plus multiplier * bias).
// 16-byte loads, all of a thread's loads of a pass issued before the first use (one trip to L2 per 1024 columns), when the
// arrays allow it; element by element otherwise.  cw and c0 are multiples of 4.
__device__ __forceinline__ void fill_relax_params(float4* s_pm, float4* s_nm, float4* s_pk, float4* s_nk, int c0, int cw, int n,
                                                  int side, int b, const float* __restrict__ lambda, const float* __restrict__ mu,
                                                  const float* __restrict__ nu, const float* __restrict__ bias)
{
    const bool vec = (n & 3) == 0 && (!lambda || ((((uintptr_t)(lambda + (size_t)b * n)) | ((uintptr_t)(mu + (size_t)b * n)) |
                                                   ((uintptr_t)(nu + (size_t)b * n))) & 15) == 0) &&
                     (!bias || (((uintptr_t)bias) & 15) == 0);
    if (vec) {
        const int n4 = n >> 2, c04 = c0 >> 2, cw4 = cw >> 2;
        const float4* la4 = reinterpret_cast<const float4*>(lambda ? lambda + (size_t)b * n : nullptr);
        const float4* mu4 = reinterpret_cast<const float4*>(mu ? mu + (size_t)b * n : nullptr);
        const float4* nu4 = reinterpret_cast<const float4*>(nu ? nu + (size_t)b * n : nullptr);
        const float4* bi4 = reinterpret_cast<const float4*>(bias);
        for (int i4 = threadIdx.x; i4 < cw4; i4 += kThreads) {
            float4 la = make_float4(1.f, 1.f, 1.f, 1.f), m = la, v = make_float4(0.f, 0.f, 0.f, 0.f), bj = v;
            const bool live = c04 + i4 < n4;
            if (live) {
                if (lambda) { la = la4[c04 + i4]; m = mu4[c04 + i4]; v = nu4[c04 + i4]; }
                if (bias) bj = bi4[c04 + i4];
            }
            const float lav[4] = {la.x, la.y, la.z, la.w}, mv[4] = {m.x, m.y, m.z, m.w};
            const float vv[4] = {v.x, v.y, v.z, v.w}, bv[4] = {bj.x, bj.y, bj.z, bj.w};
            float pm[4], nm[4], pk[4], nk[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                pm[e] = live ? (side == 0 ? lav[e] : mv[e]) : 0.f;      // lower rows: C >= 0 takes L, C < 0 takes U
                nm[e] = live ? (side == 0 ? mv[e] : lav[e]) : 0.f;
                pk[e] = live ? (side == 0 ? 0.0f : vv[e]) + pm[e] * bv[e] : 0.f;
                nk[e] = live ? (side == 0 ? vv[e] : 0.0f) + nm[e] * bv[e] : 0.f;
            }
            s_pm[i4] = make_float4(pm[0], pm[1], pm[2], pm[3]);
            s_nm[i4] = make_float4(nm[0], nm[1], nm[2], nm[3]);
            s_pk[i4] = make_float4(pk[0], pk[1], pk[2], pk[3]);
            s_nk[i4] = make_float4(nk[0], nk[1], nk[2], nk[3]);
        }
    } else {
        for (int i = threadIdx.x; i < cw; i += kThreads) {
            const int col = c0 + i;
            float pm = 0.f, nm = 0.f, pk = 0.f, nk = 0.f;
            if (col < n) {
                const float la = lambda ? lambda[(size_t)b * n + col] : 1.0f;
                const float m = mu ? mu[(size_t)b * n + col] : 1.0f;
                const float v = nu ? nu[(size_t)b * n + col] : 0.0f;
                const float bj = bias ? bias[col] : 0.0f;
                pm = side == 0 ? la : m;
                nm = side == 0 ? m : la;
                pk = (side == 0 ? 0.0f : v) + pm * bj;
                nk = (side == 0 ? v : 0.0f) + nm * bj;
            }
            reinterpret_cast<float*>(s_pm)[i] = pm;
            reinterpret_cast<float*>(s_nm)[i] = nm;
            reinterpret_cast<float*>(s_pk)[i] = pk;
            reinterpret_cast<float*>(s_nk)[i] = nk;
        }
    }
}

// The box of input b for columns [c0, c0 + cw) into LDS: the bound a coefficient >= 0 takes, the bound a negative one takes.
__device__ __forceinline__ void fill_box_params(float4* s_p, float4* s_n, int c0, int cw, int n, int side, int b,
                                                const float* __restrict__ lo, const float* __restrict__ hi)
{
    const bool vec = (n & 3) == 0 && ((((uintptr_t)(lo + (size_t)b * n)) | ((uintptr_t)(hi + (size_t)b * n))) & 15) == 0;
    if (vec) {
        const int n4 = n >> 2, c04 = c0 >> 2, cw4 = cw >> 2;
        const float4* lo4 = reinterpret_cast<const float4*>(lo + (size_t)b * n);
        const float4* hi4 = reinterpret_cast<const float4*>(hi + (size_t)b * n);
        for (int i4 = threadIdx.x; i4 < cw4; i4 += kThreads) {
            float4 lv = make_float4(0.f, 0.f, 0.f, 0.f), hv = lv;
            if (c04 + i4 < n4) { lv = lo4[c04 + i4]; hv = hi4[c04 + i4]; }
            const bool lower = side == 0;
            s_p[i4] = make_float4(lower ? lv.x : hv.x, lower ? lv.y : hv.y, lower ? lv.z : hv.z, lower ? lv.w : hv.w);
            s_n[i4] = make_float4(lower ? hv.x : lv.x, lower ? hv.y : lv.y, lower ? hv.z : lv.z, lower ? hv.w : lv.w);
        }
    } else {
        for (int i = threadIdx.x; i < cw; i += kThreads) {
            const int col = c0 + i;
            float pv = 0.f, qv = 0.f;
            if (col < n) {
                const float lv = lo[(size_t)b * n + col], hv = hi[(size_t)b * n + col];
                pv = side == 0 ? lv : hv;
                qv = side == 0 ? hv : lv;
            }
            reinterpret_cast<float*>(s_p)[i] = pv;
            reinterpret_cast<float*>(s_n)[i] = qv;
        }
    }
}

// Sign-split ReLU step + bias fold (replace_lower / replace_upper through a ReLU layer, then the
// constant part of the affine layer below) for rows of any width.  grid = (row tiles, nsides*batch).  The per-input
// parameters are staged in LDS a chunk of columns at a time.  A wavefront streams two rows at a time so that up to
// eight 16-byte loads per lane are in flight.
template <bool SHARED>
__global__ __launch_bounds__(kThreads) void relax_step_kernel(
    float* __restrict__ C, int ldc, double* __restrict__ cst, int batch, int R, int n,
    const float* __restrict__ lambda, const float* __restrict__ mu, const float* __restrict__ nu,
    const float* __restrict__ bias, const float* __restrict__ src, int ld_src,
    const float* __restrict__ cst_init, int rows_per_wave, int chunk)
{
    extern __shared__ float4 s_par[];                  // [4][chunk/4]: pm, nm, pk, nk
    const int ch4 = chunk >> 2;
    float4* s_pm = s_par;
    float4* s_nm = s_par + ch4;
    float4* s_pk = s_par + 2 * ch4;
    float4* s_nk = s_par + 3 * ch4;
    const int sb = blockIdx.y;
    const int side = sb / batch, b = sb - side * batch;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r0 = blockIdx.x * (rows_per_wave * kWaves) + wave * rows_per_wave;

    double acc[kMaxRowsPerWave];
#pragma unroll
    for (int q = 0; q < kMaxRowsPerWave; ++q) acc[q] = 0.0;

    for (int c0 = 0; c0 < ldc; c0 += chunk) {
        const int cw = min(chunk, ldc - c0);           // multiple of 4 (ldc is)
        if (c0 > 0) __syncthreads();
        fill_relax_params(s_pm, s_nm, s_pk, s_nk, c0, cw, n, side, b, lambda, mu, nu, bias);
        __syncthreads();
        const int cw4 = cw >> 2;
        const int nloc = n - c0;
#pragma unroll
        for (int qp = 0; qp < kMaxRowsPerWave; qp += 2) {
            if (qp >= rows_per_wave || r0 + qp >= R) break;
            const bool two = qp + 1 < rows_per_wave && r0 + qp + 1 < R;
            const float4* in[2];
            float4* out[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int r = r0 + qp + ((h == 1 && two) ? 1 : 0);
                const size_t m = (size_t)sb * R + r;
                in[h] = reinterpret_cast<const float4*>(SHARED ? src + (size_t)r * ld_src + c0 : C + m * ldc + c0);
                out[h] = reinterpret_cast<float4*>(C + m * ldc + c0);
            }
            double a[2] = {0.0, 0.0};
            for (int base = 0; base < cw4; base += 64 * 4) {
                float4 v[2][4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int i4 = base + t * 64 + lane;
                    if (i4 < cw4) {
                        v[0][t] = SHARED ? in[0][i4] : in[0][i4];
                        if (two) v[1][t] = SHARED ? in[1][i4] : in[1][i4];
                    }
                }
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int i4 = base + t * 64 + lane;
                    if (i4 >= cw4) continue;
                    const float4 pm = s_pm[i4], nm = s_nm[i4], pk = s_pk[i4], nk = s_nk[i4];
                    const float pmv[4] = {pm.x, pm.y, pm.z, pm.w}, nmv[4] = {nm.x, nm.y, nm.z, nm.w};
                    const float pkv[4] = {pk.x, pk.y, pk.z, pk.w}, nkv[4] = {nk.x, nk.y, nk.z, nk.w};
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        if (h == 1 && !two) break;
                        const float x[4] = {v[h][t].x, v[h][t].y, v[h][t].z, v[h][t].w};
                        float y[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const bool pos = x[e] >= 0.0f;
                            const bool live = i4 * 4 + e < nloc;     // padding columns come out as exact zeros
                            y[e] = live ? x[e] * (pos ? pmv[e] : nmv[e]) : 0.0f;
                            a[h] = live ? fmaf(x[e], pos ? pkv[e] : nkv[e], a[h]) : a[h];
                        }
                        *(out[h] + i4) = make_float4(y[0], y[1], y[2], y[3]);
                    }
                }
            }
            acc[qp] += a[0];
            acc[qp + 1] += a[1];
        }
    }
#pragma unroll
    for (int q = 0; q < kMaxRowsPerWave; ++q) {
        const int r = r0 + q;
        if (q >= rows_per_wave || r >= R) break;
        const double t = wave_sum(acc[q]);
        if (lane == 0) {
            const size_t m = (size_t)sb * R + r;
            cst[m] = (cst_init ? (double)cst_init[r] : cst[m]) + t;
        }
    }
}

// Concretisation (simplify_lower / simplify_upper): one wavefront per two rows, box of input b in LDS.
template <bool SHARED>
__global__ __launch_bounds__(kThreads) void concretise_kernel(
    const float* __restrict__ C, int ldc, const double* __restrict__ cst, int batch, int R, int n,
    const float* __restrict__ lo, const float* __restrict__ hi, float* __restrict__ out_l,
    float* __restrict__ out_u, const float* __restrict__ src, int ld_src,
    const float* __restrict__ cst_init, int rows_per_wave, int chunk,
    const float* __restrict__ part, int nslots, long long part_stride)
{
    extern __shared__ float4 s_par[];                  // [2][chunk/4]: bound taken by C >= 0 / C < 0
    float4* s_p = s_par;
    float4* s_n = s_par + (chunk >> 2);
    const int sb = blockIdx.y;
    const int side = sb / batch, b = sb - side * batch;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r0 = blockIdx.x * (rows_per_wave * kWaves) + wave * rows_per_wave;

    double acc[kMaxRowsPerWave];
#pragma unroll
    for (int q = 0; q < kMaxRowsPerWave; ++q) acc[q] = 0.0;

    for (int c0 = 0; c0 < ldc; c0 += chunk) {
        const int cw = min(chunk, ldc - c0);
        if (c0 > 0) __syncthreads();
        fill_box_params(s_p, s_n, c0, cw, n, side, b, lo, hi);
        __syncthreads();
        const int cw4 = cw >> 2;
        const int nloc = n - c0;
#pragma unroll
        for (int qp = 0; qp < kMaxRowsPerWave; qp += 2) {
            if (qp >= rows_per_wave || r0 + qp >= R) break;
            const bool two = qp + 1 < rows_per_wave && r0 + qp + 1 < R;
            const float4* in[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int r = r0 + qp + ((h == 1 && two) ? 1 : 0);
                const size_t m = (size_t)sb * R + r;
                in[h] = reinterpret_cast<const float4*>(SHARED ? src + (size_t)r * ld_src + c0 : C + m * ldc + c0);
            }
            double a[2] = {0.0, 0.0};
            for (int base = 0; base < cw4; base += 64 * 4) {
                float4 v[2][4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int i4 = base + t * 64 + lane;
                    if (i4 < cw4) {
                        v[0][t] = SHARED ? in[0][i4] : in[0][i4];
                        if (two) v[1][t] = SHARED ? in[1][i4] : in[1][i4];
                    }
                }
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int i4 = base + t * 64 + lane;
                    if (i4 >= cw4) continue;
                    const float4 p = s_p[i4], ng = s_n[i4];
                    const float pv[4] = {p.x, p.y, p.z, p.w}, nv[4] = {ng.x, ng.y, ng.z, ng.w};
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        if (h == 1 && !two) break;
                        const float x[4] = {v[h][t].x, v[h][t].y, v[h][t].z, v[h][t].w};
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (i4 * 4 + e < nloc) a[h] += (double)x[e] * (double)(x[e] >= 0.0f ? pv[e] : nv[e]);
                    }
                }
            }
            acc[qp] += a[0];
            acc[qp + 1] += a[1];
        }
    }
#pragma unroll
    for (int q = 0; q < kMaxRowsPerWave; ++q) {
        const int r = r0 + q;
        if (q >= rows_per_wave || r >= R) break;
        const size_t m = (size_t)sb * R + r;
        double extra = 0.0;        // row-constant partial sums left by fused contraction epilogues, slot order fixed
        for (int t = lane; t < nslots; t += 64) extra += (double)part[(size_t)t * part_stride + m];
        const double t = wave_sum(acc[q] + extra);
        if (lane == 0) {
            const double v = (cst_init ? (double)cst_init[r] : cst[m]) + t;
            (side == 0 ? out_l : out_u)[(size_t)b * R + r] = (float)v;
        }
    }
}

// Streaming kernels for rows whose per-input parameters fit LDS whole (rows of up to 2048 columns: at most 32 KB for the sign-split
// ReLU step, 16 KB for the concretisation, so that five or more workgroups fit a compute unit; wider rows go to the
// kernels above, which walk chunks of 2048 columns and were measured faster there).  Many short workgroups, in row order: a wavefront's work is
// a unit (pair of rows, segment of 1024 columns) -- one 16-byte load per lane covers a quarter of a segment, a pair
// shares every LDS read of the parameters -- and with the default launch shape a wavefront owns ONE pair.  Its loads are
// issued before the group's parameters are staged, and the staging itself is one trip to L2 (16-byte loads, all issued
// before the first use).  Measured on gfx950: fewer, longer-lived workgroups that walk many pairs (parameters staged once
// per group, next unit's loads in flight under the current one) were slower at every shape -- the rate of these passes
// follows the number of resident wavefronts, not the depth of a wavefront's own queue.  Per-lane partial sums of a
// segment (at most 16 products) are fp32; they are added up per row in fp64, lanes are combined in fp64 by wave shuffles.
// Pairs of a group are dealt round-robin to the wavefronts of all its workgroups.
constexpr int kSeg4 = 256;             // float4 per segment of a row (1024 columns)

// NT: the rows are read and written with non-temporal accesses.  Measured: better when the rows are larger than the 256 MB
// Infinity Cache (1 GB of rows: 0.71 against 0.68 of the HBM rate), worse when a following kernel could still find them
// there (100-270 MB: 0.66-0.72 against 0.72-0.74); the launcher picks by size.  The kernels that walk wide rows in chunks use
// plain accesses (measured better at both of their shapes), the streaming concretisation non-temporal loads (better at both).
template <bool SHARED, bool NT>
__global__ __launch_bounds__(kThreads) void relax_step_stream_kernel(
    float* __restrict__ C, int ldc, double* __restrict__ cst, int batch, int R, int n,
    const float* __restrict__ lambda, const float* __restrict__ mu, const float* __restrict__ nu,
    const float* __restrict__ bias, const float* __restrict__ src, int ld_src,
    const float* __restrict__ cst_init, int rows_per_block)
{
    extern __shared__ float4 s_par[];                  // [4][ldc/4]: pm, nm, pk, nk
    const int cw4 = ldc >> 2;
    float4* s_pm = s_par;
    float4* s_nm = s_par + cw4;
    float4* s_pk = s_par + 2 * cw4;
    float4* s_nk = s_par + 3 * cw4;
    const int sb = blockIdx.y;
    const int side = sb / batch, b = sb - side * batch;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    // pairs of the group are dealt round-robin to all wavefronts of all its workgroups, so that at any time the group's
    // workgroups read one compact window of rows
    const int rbeg = 0, rend = R;
    const int npairs = (R + 1) >> 1;
    const int first = blockIdx.x * kWaves + wave, stride = gridDim.x * kWaves;
    const int nseg = (cw4 + kSeg4 - 1) / kSeg4;
    const int nunits = npairs > first ? ((npairs - first + stride - 1) / stride) * nseg : 0;   // of this wavefront

    auto row_of = [&](int p, int h) { const int r = rbeg + 2 * p + h; return r < rend ? r : rend - 1; };
    auto load_unit = [&](int k, float4 (&v)[2][4]) {
        const int p = first + (k / nseg) * stride, base = (k % nseg) * kSeg4;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int r = row_of(p, h);
            const float4* in = reinterpret_cast<const float4*>(SHARED ? src + (size_t)r * ld_src
                                                                      : C + ((size_t)sb * R + r) * ldc);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int i4 = base + t * 64 + lane;
                if (i4 < cw4) v[h][t] = (SHARED || !NT) ? in[i4] : nt_load4(in + i4);
            }
        }
    };
    double ad[2] = {0.0, 0.0};
    auto compute_unit = [&](int k, float4 (&v)[2][4]) {
        const int p = first + (k / nseg) * stride, seg = k % nseg, base = seg * kSeg4;
        float a[2] = {0.0f, 0.0f};
        const bool two = rbeg + 2 * p + 1 < rend;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int i4 = base + t * 64 + lane;
            if (i4 >= cw4) continue;
            const float4 pm = s_pm[i4], nm = s_nm[i4], pk = s_pk[i4], nk = s_nk[i4];
            const float pmv[4] = {pm.x, pm.y, pm.z, pm.w}, nmv[4] = {nm.x, nm.y, nm.z, nm.w};
            const float pkv[4] = {pk.x, pk.y, pk.z, pk.w}, nkv[4] = {nk.x, nk.y, nk.z, nk.w};
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (h == 1 && !two) break;
                const float x[4] = {v[h][t].x, v[h][t].y, v[h][t].z, v[h][t].w};
                float y[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool pos = x[e] >= 0.0f;
                    const bool live = i4 * 4 + e < n;        // padding columns come out as exact zeros
                    y[e] = live ? x[e] * (pos ? pmv[e] : nmv[e]) : 0.0f;
                    a[h] = live ? fmaf(x[e], pos ? pkv[e] : nkv[e], a[h]) : a[h];
                }
                const size_t m = (size_t)sb * R + row_of(p, h);
                if constexpr (NT) nt_store4(reinterpret_cast<float4*>(C + m * ldc) + i4, y[0], y[1], y[2], y[3]);
                else reinterpret_cast<float4*>(C + m * ldc)[i4] = make_float4(y[0], y[1], y[2], y[3]);
            }
        }
        ad[0] += (double)a[0];
        ad[1] += (double)a[1];
        if (seg != nseg - 1) return;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            if (h == 1 && !two) break;
            const double t = wave_sum(ad[h]);
            if (lane == 0) {
                const int r = row_of(p, h);
                const size_t m = (size_t)sb * R + r;
                cst[m] = (cst_init ? (double)cst_init[r] : cst[m]) + t;
            }
        }
        ad[0] = ad[1] = 0.0;
    };

    float4 va[2][4];
    if (nunits > 0) load_unit(0, va);
    fill_relax_params(s_pm, s_nm, s_pk, s_nk, 0, ldc, n, side, b, lambda, mu, nu, bias);
    __syncthreads();
    for (int k = 0; k < nunits; ++k) {
        if (k > 0) load_unit(k, va);
        compute_unit(k, va);
    }
}

template <bool SHARED>
__global__ __launch_bounds__(kThreads) void concretise_stream_kernel(
    const float* __restrict__ C, int ldc, const double* __restrict__ cst, int batch, int R, int n,
    const float* __restrict__ lo, const float* __restrict__ hi, float* __restrict__ out_l,
    float* __restrict__ out_u, const float* __restrict__ src, int ld_src,
    const float* __restrict__ cst_init, int rows_per_block,
    const float* __restrict__ part, int nslots, long long part_stride)
{
    extern __shared__ float4 s_par[];                  // [2][ldc/4]
    const int cw4 = ldc >> 2;
    float4* s_p = s_par;
    float4* s_n = s_par + cw4;
    const int sb = blockIdx.y;
    const int side = sb / batch, b = sb - side * batch;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    // pairs of the group are dealt round-robin to all wavefronts of all its workgroups, so that at any time the group's
    // workgroups read one compact window of rows
    const int rbeg = 0, rend = R;
    const int npairs = (R + 1) >> 1;
    const int first = blockIdx.x * kWaves + wave, stride = gridDim.x * kWaves;
    const int nseg = (cw4 + kSeg4 - 1) / kSeg4;
    const int nunits = npairs > first ? ((npairs - first + stride - 1) / stride) * nseg : 0;   // of this wavefront

    auto row_of = [&](int p, int h) { const int r = rbeg + 2 * p + h; return r < rend ? r : rend - 1; };
    auto load_unit = [&](int k, float4 (&v)[2][4]) {
        const int p = first + (k / nseg) * stride, base = (k % nseg) * kSeg4;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int r = row_of(p, h);
            const float4* in = reinterpret_cast<const float4*>(SHARED ? src + (size_t)r * ld_src
                                                                      : C + ((size_t)sb * R + r) * ldc);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int i4 = base + t * 64 + lane;
                if (i4 < cw4) v[h][t] = SHARED ? in[i4] : nt_load4(in + i4);
            }
        }
    };
    double ad[2] = {0.0, 0.0};
    auto compute_unit = [&](int k, float4 (&v)[2][4]) {
        const int p = first + (k / nseg) * stride, seg = k % nseg, base = seg * kSeg4;
        float a[2] = {0.0f, 0.0f};
        const bool two = rbeg + 2 * p + 1 < rend;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int i4 = base + t * 64 + lane;
            if (i4 >= cw4) continue;
            const float4 pp = s_p[i4], ng = s_n[i4];
            const float pv[4] = {pp.x, pp.y, pp.z, pp.w}, nv[4] = {ng.x, ng.y, ng.z, ng.w};
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (h == 1 && !two) break;
                const float x[4] = {v[h][t].x, v[h][t].y, v[h][t].z, v[h][t].w};
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (i4 * 4 + e < n) a[h] = fmaf(x[e], x[e] >= 0.0f ? pv[e] : nv[e], a[h]);
            }
        }
        ad[0] += (double)a[0];
        ad[1] += (double)a[1];
        if (seg != nseg - 1) return;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            if (h == 1 && !two) break;
            const int r = row_of(p, h);
            const size_t m = (size_t)sb * R + r;
            double extra = 0.0;
            for (int t = lane; t < nslots; t += 64) extra += (double)part[(size_t)t * part_stride + m];
            const double t = wave_sum(ad[h] + extra);
            if (lane == 0) {
                const double val = (cst_init ? (double)cst_init[r] : cst[m]) + t;
                (side == 0 ? out_l : out_u)[(size_t)b * R + r] = (float)val;
            }
        }
        ad[0] = ad[1] = 0.0;
    };

    float4 va[2][4];
    if (nunits > 0) load_unit(0, va);
    fill_box_params(s_p, s_n, 0, ldc, n, side, b, lo, hi);
    __syncthreads();
    for (int k = 0; k < nunits; ++k) {
        if (k > 0) load_unit(k, va);
        compute_unit(k, va);
    }
}

// Packed parameters of the sign-split ReLU step for both sides (see launch_pack_relax).
__global__ __launch_bounds__(kThreads) void pack_relax_kernel(
    const float* __restrict__ lambda, const float* __restrict__ mu, const float* __restrict__ nu,
    const float* __restrict__ bias, int batch, int n, int ld, float4* __restrict__ pk)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;       // over [2][batch][ld]
    if (i >= (int64_t)2 * batch * ld) return;
    const int col = (int)(i % ld);
    const int sb = (int)(i / ld);
    const int side = sb / batch, b = sb - side * batch;
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
    if (col < n) {
        const float la = lambda[(size_t)b * n + col], m = mu[(size_t)b * n + col], v = nu[(size_t)b * n + col];
        const float bj = bias ? bias[col] : 0.0f;
        o.x = side == 0 ? la : m;
        o.y = side == 0 ? m : la;
        o.z = (side == 0 ? 0.0f : v) + o.x * bj;
        o.w = (side == 0 ? v : 0.0f) + o.y * bj;
    }
    pk[i] = o;
}

// Sum of two blocks of one expression that have reached the same layer (residual networks: the rows that went
// through a block's branch and the rows that waited on its skip connection).  The waiting block covers a
// sub-window of the rows' patch (or all of a dense row: one position with n "channels"):
//   kind 0: a block of its own per row, src[m][ph1*pw1*C];  kind 1: one block per output channel of the bounded
//   layer, shared by all inputs and positions, src[r % rows_C][...];  kind 2: coefficient 1 on the row's own neuron.
struct MergeArgs {
    float* dst; int ld_dst;
    const float* src; int ld_src;
    int R, rows_C;
    int ph1, pw1, pw2, C, d;      // waiting block ph1 x pw1 x C sits at offset (d, d) inside rows of width pw2
    int kind;
};

__global__ __launch_bounds__(kThreads) void merge_block_kernel(MergeArgs a)
{
    const size_t m = blockIdx.x;
    const int r = (int)(m % (size_t)a.R);
    float* dst = a.dst + m * a.ld_dst;
    if (a.kind == 2) {
        if (threadIdx.x == 0) dst[(size_t)(a.d * a.pw2 + a.d) * a.C + r % a.rows_C] += 1.0f;
        return;
    }
    const float* src = a.src + (a.kind == 1 ? (size_t)(r % a.rows_C) : m) * a.ld_src;
    const int n1 = a.ph1 * a.pw1 * a.C;
    for (int e = threadIdx.x; e < n1; e += kThreads) {
        const int pos = e / a.C, c = e - pos * a.C;
        const int py = pos / a.pw1, px = pos - py * a.pw1;
        dst[(size_t)((py + a.d) * a.pw2 + px + a.d) * a.C + c] += src[e];
    }
}

// Concretisation of a waiting block against the stored bounds of the layer it is over, added to the rows' constants
// (a depth-limited traversal that ends while a block still waits on a skip connection: simplify_* maps over the
// terms of both layers).  One wavefront per row; the block kinds are those of merge_block_kernel.
struct BlockBoundArgs {
    double* cst;
    const float* src; int ld_src;
    const float* lo; const float* hi;      // [batch][n] bounds of the block's layer
    long long M; int R, rows_C, rows_W, batch, nsides, n;
    int patch, ph, pw, C, S, P, gh, gw;    // patch geometry of the block (patch != 0)
    int kind;
};

__global__ __launch_bounds__(kThreads) void block_bound_kernel(BlockBoundArgs a)
{
    const long long m = (long long)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (m >= a.M) return;
    const int lane = threadIdx.x & 63;
    const int g = (int)(m / a.R), r = (int)(m - (long long)g * a.R);
    const int side = a.nsides == 1 ? 0 : (g >= a.batch), b = g - (g >= a.batch ? a.batch : 0);
    const float* lo = a.lo + (size_t)b * a.n;
    const float* hi = a.hi + (size_t)b * a.n;
    double acc = 0.0;
    if (a.kind == 2) {
        if (lane == 0) acc = side == 0 ? lo[r] : hi[r];                  // coefficient 1 on the row's own neuron
    } else {
        const float* src = a.src + (a.kind == 1 ? (size_t)(r % a.rows_C) : (size_t)m) * a.ld_src;
        const int n1 = a.patch ? a.ph * a.pw * a.C : a.n;
        const int wo = (r / a.rows_C) % a.rows_W, ho = r / (a.rows_C * a.rows_W);
        const int oy = ho * a.S - a.P, ox = wo * a.S - a.P;
        for (int e = lane; e < n1; e += 64) {
            int idx = e;
            if (a.patch) {
                const int pos = e / a.C, c = e - pos * a.C;
                const int py = pos / a.pw, px = pos - py * a.pw;
                const int gy = oy + py, gx = ox + px;
                if (gy < 0 || gy >= a.gh || gx < 0 || gx >= a.gw) continue;     // zero padding: no neuron there
                idx = (gy * a.gw + gx) * a.C + c;
            }
            const float x = src[e];
            acc += (double)x * (double)((x >= 0.0f) == (side == 0) ? lo[idx] : hi[idx]);
        }
    }
    acc = wave_sum(acc);
    if (lane == 0) a.cst[m] += acc;
}

// Compact parameters of a ReLU layer for kernels that apply the sign split themselves: (mu, nu) per (input, neuron)
// with lambda (0 or 1) carried in the sign bit of nu (nu itself is never negative); columns n..ld-1 zero.
__global__ __launch_bounds__(kThreads) void pack_relax2_kernel(
    const float* __restrict__ lambda, const float* __restrict__ mu, const float* __restrict__ nu, int batch, int n, int ld,
    float2* __restrict__ pk2)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;       // over [batch][ld]
    if (i >= (int64_t)batch * ld) return;
    const int col = (int)(i % ld), b = (int)(i / ld);
    float2 o = make_float2(0.f, 0.f);
    if (col < n) {
        const float v = fabsf(nu[(size_t)b * n + col]);
        o.x = mu[(size_t)b * n + col];
        o.y = lambda[(size_t)b * n + col] != 0.0f ? -v : v;
    }
    pk2[i] = o;
}

// relax_params_kernel, pack_relax_kernel and pack_relax2_kernel in one launch (the same arithmetic, value by value):
// one thread per (input, padded column); pk and pk2 may be NULL.
__global__ __launch_bounds__(kThreads) void relax_params_pack_kernel(
    const float* __restrict__ l, const float* __restrict__ u, float* __restrict__ lambda, float* __restrict__ mu,
    float* __restrict__ nu, float* __restrict__ rl, float* __restrict__ ru, const float* __restrict__ bias, int batch, int n,
    int ld, float4* __restrict__ pk, float2* __restrict__ pk2)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;       // over [batch][ld]
    if (i >= (int64_t)batch * ld) return;
    const int col = (int)(i % ld), b = (int)(i / ld);
    float4 lo4 = make_float4(0.f, 0.f, 0.f, 0.f), up4 = lo4;
    float2 o2 = make_float2(0.f, 0.f);
    if (col < n) {
        const size_t k = (size_t)b * n + col;
        const float lv = l[k], uv = u[k];
        const float la = (lv + uv >= 0.0f) ? 1.0f : 0.0f;
        float m, v;
        if (lv >= 0.0f) { m = 1.0f; v = 0.0f; }
        else if (uv <= 0.0f) { m = 0.0f; v = 0.0f; }
        else {
            const float d = uv - lv;
            m = uv / d;
            v = -(uv * lv) / d;
        }
        lambda[k] = la;
        mu[k] = m;
        nu[k] = v;
        rl[k] = lv >= 0.0f ? lv : 0.0f;
        ru[k] = uv >= 0.0f ? uv : 0.0f;
        const float bj = bias ? bias[col] : 0.0f;
        lo4 = make_float4(la, m, 0.0f + la * bj, v + m * bj);          // lower side: (lambda, mu | ., nu)
        up4 = make_float4(m, la, v + m * bj, 0.0f + la * bj);          // upper side: (mu, lambda | nu, .)
        const float av = fabsf(v);
        o2 = make_float2(m, la != 0.0f ? -av : av);
    }
    if (pk) {
        pk[i] = lo4;
        pk[(size_t)batch * ld + i] = up4;
    }
    if (pk2) pk2[i] = o2;
}

__global__ __launch_bounds__(kThreads) void pack_bounds_kernel(
    const float* __restrict__ lo, const float* __restrict__ hi, int batch, int n, int ld, float4* __restrict__ pk)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= (int64_t)2 * batch * ld) return;
    const int col = (int)(i % ld);
    const int sb = (int)(i / ld);
    const int side = sb / batch, b = sb - side * batch;
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
    if (col < n) {
        const float lv = lo[(size_t)b * n + col], hv = hi[(size_t)b * n + col];
        o.z = side == 0 ? lv : hv;
        o.w = side == 0 ? hv : lv;
    }
    pk[i] = o;
}

__global__ __launch_bounds__(kThreads) void finalize_bounds_kernel(
    const double* __restrict__ cst, const float* __restrict__ part, int nslots, long long part_stride, int batch, int R,
    long long M, float* __restrict__ out_l, float* __restrict__ out_u)
{
    const long long m = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (m >= M) return;
    double v = cst[m];
    // eight slots requested at a time, added in index order (the loads are independent, the sum is not reordered)
    int t = 0;
    for (; t + 8 <= nslots; t += 8) {
        float p[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) p[k] = part[(size_t)(t + k) * part_stride + m];
#pragma unroll
        for (int k = 0; k < 8; ++k) v += (double)p[k];
    }
    for (; t < nslots; ++t) v += (double)part[(size_t)t * part_stride + m];
    const long long sb = m / R;
    const int r = (int)(m - sb * R);
    const int side = (int)(sb / batch), b = (int)(sb - (long long)side * batch);
    (side == 0 ? out_l : out_u)[(size_t)b * R + r] = (float)v;
}

// The constant + the partial sums of row m, slots added in index order (finalize_bounds_kernel's order).
__device__ __forceinline__ float folded_bound(const double* __restrict__ cst, const float* __restrict__ part, int nslots,
                                              long long part_stride, long long m)
{
    double v = cst[m];
    int t = 0;
    for (; t + 8 <= nslots; t += 8) {
        float p[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) p[k] = part[(size_t)(t + k) * part_stride + m];
#pragma unroll
        for (int k = 0; k < 8; ++k) v += (double)p[k];
    }
    for (; t < nslots; ++t) v += (double)part[(size_t)t * part_stride + m];
    return (float)v;
}

// finalize_bounds_kernel for an affine layer (both sides, R = n rows per group) and relax_params_pack_kernel for the ReLU
// layer above it in one launch, value by value the same arithmetic: one thread per (input, padded column).
__global__ __launch_bounds__(kThreads) void finalize_relax_pack_kernel(
    const double* __restrict__ cst, const float* __restrict__ part, int nslots, long long part_stride,
    float* __restrict__ out_l, float* __restrict__ out_u, float* __restrict__ lambda, float* __restrict__ mu,
    float* __restrict__ nu, float* __restrict__ rl, float* __restrict__ ru, const float* __restrict__ bias, int batch, int n,
    int ld, float4* __restrict__ pk, float2* __restrict__ pk2)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;       // over [batch][ld]
    if (i >= (int64_t)batch * ld) return;
    const int col = (int)(i % ld), b = (int)(i / ld);
    float4 lo4 = make_float4(0.f, 0.f, 0.f, 0.f), up4 = lo4;
    float2 o2 = make_float2(0.f, 0.f);
    if (col < n) {
        const size_t k = (size_t)b * n + col;
        const float lv = folded_bound(cst, part, nslots, part_stride, (long long)b * n + col);
        const float uv = folded_bound(cst, part, nslots, part_stride, ((long long)batch + b) * n + col);
        out_l[k] = lv;
        out_u[k] = uv;
        const float la = (lv + uv >= 0.0f) ? 1.0f : 0.0f;
        float m, v;
        if (lv >= 0.0f) { m = 1.0f; v = 0.0f; }
        else if (uv <= 0.0f) { m = 0.0f; v = 0.0f; }
        else {
            const float d = uv - lv;
            m = uv / d;
            v = -(uv * lv) / d;
        }
        lambda[k] = la;
        mu[k] = m;
        nu[k] = v;
        rl[k] = lv >= 0.0f ? lv : 0.0f;
        ru[k] = uv >= 0.0f ? uv : 0.0f;
        const float bj = bias ? bias[col] : 0.0f;
        lo4 = make_float4(la, m, 0.0f + la * bj, v + m * bj);
        up4 = make_float4(m, la, v + m * bj, 0.0f + la * bj);
        const float av = fabsf(v);
        o2 = make_float2(m, la != 0.0f ? -av : av);
    }
    if (pk) {
        pk[i] = lo4;
        pk[(size_t)batch * ld + i] = up4;
    }
    if (pk2) pk2[i] = o2;
}

// finalize_bounds_kernel and split_final_kernel for the merged last pass in one launch: one wavefront per input, lane r
// takes row r of the input's two groups (Rs <= 64 rows each).
__global__ __launch_bounds__(64) void finalize_split_final_kernel(
    const double* __restrict__ cst, const float* __restrict__ part, int nslots, long long part_stride, int batch, int nK, int Rs,
    float* __restrict__ l, float* __restrict__ u, float* __restrict__ margin, int32_t* __restrict__ verdict)
{
    const int b = blockIdx.x, r = threadIdx.x;
    const int Rm = 2 * nK - 1;
    bool fails = false;
    if (r < Rm) {
        const float lv = folded_bound(cst, part, nslots, part_stride, (long long)b * Rs + r);
        if (r < nK) {
            l[(size_t)b * nK + r] = lv;
            u[(size_t)b * nK + r] = folded_bound(cst, part, nslots, part_stride, ((long long)batch + b) * Rs + r);
        } else {
            margin[(size_t)b * (nK - 1) + (r - nK)] = lv;
            fails = !(lv > 0.0f);
        }
    }
    const unsigned long long any = __ballot(fails);
    if (r == 0) verdict[b] = any == 0ull ? 1 : 0;
}

__global__ __launch_bounds__(kThreads) void margin_rows_kernel(
    const float* __restrict__ W, int ldw, const float* __restrict__ bias, const int32_t* __restrict__ label,
    int nK, int n, float* __restrict__ C, int ldc, double* __restrict__ cst)
{
    const int m = blockIdx.x;                // b * (nK-1) + q
    const int b = m / (nK - 1), q = m - b * (nK - 1);
    const int t = min(max(label[b], 0), nK - 1);       // labels are validated while this runs: never index out of range
    const int o = q < t ? q : q + 1;
    for (int i = threadIdx.x; i < ldc; i += kThreads)
        C[(size_t)m * ldc + i] = i < n ? W[(size_t)t * ldw + i] - W[(size_t)o * ldw + i] : 0.0f;
    if (threadIdx.x == 0) cst[m] = (double)bias[t] - (double)bias[o];
}

// Rows of the last pass when output-layer bounds and margins share one traversal: for group (side, b),
// rows 0..nK-1 are the output neurons' own expressions (weight rows, bias), rows nK..2nK-2 the margin
// expressions logit[label_b] - logit[o] for the nK-1 other classes o in ascending order.  A group holds Rs >= 2nK-1
// rows; rows past 2nK-2 are zero (padding that lets the pass use kernels with a minimum group size).
__global__ __launch_bounds__(kThreads) void final_rows_kernel(
    const float* __restrict__ W, int ldw, const float* __restrict__ bias, const int32_t* __restrict__ label, int batch,
    int nK, int n, float* __restrict__ C, int ldc, double* __restrict__ cst, int Rs)
{
    const int Rm = 2 * nK - 1;
    const int m = blockIdx.x;                 // (side*batch + b)*Rs + r
    const int r = m % Rs, b = (m / Rs) % batch;
    const bool pad = r >= Rm;
    int t = pad ? 0 : r, o = -1;
    if (!pad && r >= nK) {
        const int q = r - nK;
        t = min(max(label[b], 0), nK - 1);             // labels are validated while this runs: never index out of range
        o = q < t ? q : q + 1;
    }
    for (int i = threadIdx.x; i < ldc; i += kThreads) {
        float v = 0.0f;
        if (i < n && !pad) v = o < 0 ? W[(size_t)t * ldw + i] : W[(size_t)t * ldw + i] - W[(size_t)o * ldw + i];
        C[(size_t)m * ldc + i] = v;
    }
    if (threadIdx.x == 0) cst[m] = pad ? 0.0 : o < 0 ? (double)bias[t] : (double)bias[t] - (double)bias[o];
}

// Splits the merged last pass: l,u of the output layer, margins (lower side only) and verdicts.
__global__ void split_final_kernel(const float* __restrict__ tl, const float* __restrict__ tu, int batch, int nK,
                                   float* __restrict__ l, float* __restrict__ u, float* __restrict__ margin,
                                   int32_t* __restrict__ verdict, int Rs)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    for (int r = 0; r < nK; ++r) {
        l[(size_t)b * nK + r] = tl[(size_t)b * Rs + r];
        u[(size_t)b * nK + r] = tu[(size_t)b * Rs + r];
    }
    int ok = 1;
    for (int q = 0; q < nK - 1; ++q) {
        const float mg = tl[(size_t)b * Rs + nK + q];
        margin[(size_t)b * (nK - 1) + q] = mg;
        if (!(mg > 0.0f)) ok = 0;
    }
    verdict[b] = ok;
}

__global__ void verdict_kernel(const float* __restrict__ margin, int batch, int nq, int32_t* __restrict__ verdict)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    int ok = 1;
    for (int q = 0; q < nq; ++q)
        if (!(margin[(size_t)b * nq + q] > 0.0f)) ok = 0;
    verdict[b] = ok;
}

template <bool TO_HWC>
__global__ __launch_bounds__(kThreads) void permute_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                           int batch, int Cc, int H, int W)
{
    const int64_t n = (int64_t)Cc * H * W;
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n * batch) return;
    const int64_t b = i / n;
    const int e = (int)(i - b * n);          // index in (C,H,W) order
    const int w = e % W, h = (e / W) % H, c = e / (W * H);
    const int64_t hwc = b * n + ((int64_t)h * W + w) * Cc + c;
    if (TO_HWC) dst[hwc] = src[i]; else dst[i] = src[hwc];
}


int pick_rows_per_wave(int R, int groups)
{
    if (tune(TK_ROWS_PER_WAVE) > 0) return tune(TK_ROWS_PER_WAVE);
    // Kernels that walk chunks of columns: enough blocks to cover 256 CUs a few times over, as many rows per block as
    // that allows, but at least one PAIR per wavefront (a pair shares every LDS read of the parameters: single rows
    // measured 4 % slower even where they double the number of workgroups).
    int rpw = kMaxRowsPerWave;
    while (rpw > 2 && ceil_div(R, rpw * kWaves) * groups < 2048) rpw >>= 1;
    return rpw;
}

// Rows per workgroup of the streaming kernels: one pair per wavefront; two for rows of several segments when that
// still leaves a thousand workgroups (measured: +2..4 % there, -25 % when the grid gets too small).
int pick_rows_per_block(int R, int groups, int nseg)
{
    if (tune(TK_ROWS_PER_WAVE) > 0) return tune(TK_ROWS_PER_WAVE) * kWaves;
    if (tune(TK_STREAM_WGS_PER_CU) > 0) {     // experiment: grid sized to the chip
        const int blocks_per_group = (int)std::max<int64_t>(1, (int64_t)256 * tune(TK_STREAM_WGS_PER_CU) / std::max(groups, 1));
        return (std::max((int)ceil_div(R, blocks_per_group), 2 * kWaves) + 1) & ~1;
    }
    if (nseg >= 2 && ceil_div(R, 4 * kWaves) * groups >= 1024) return 4 * kWaves;
    return 2 * kWaves;
}

}  // namespace


void launch_relax_params_pack(const float* l, const float* u, float* lambda, float* mu, float* nu, float* rl, float* ru,
                              const float* bias, int batch, int n, int ld, float* pk, float* pk2, hipStream_t s)
{
    DPC_REQUIRE(l && u && lambda && mu && nu && rl && ru && ld >= n && ((uintptr_t)pk % 16) == 0 && ((uintptr_t)pk2 % 8) == 0,
                DPC_EINVAL, "relax_params_pack: bad arguments");
    const int64_t tot = (int64_t)batch * ld;
    if (tot <= 0) return;
    hipLaunchKernelGGL(relax_params_pack_kernel, dim3((unsigned)ceil_div(tot, kThreads)), dim3(kThreads), 0, s, l, u, lambda, mu,
                       nu, rl, ru, bias, batch, n, ld, reinterpret_cast<float4*>(pk), reinterpret_cast<float2*>(pk2));
    DPC_HIP(hipGetLastError());
}

void launch_relax_params(const float* l, const float* u, float* lambda, float* mu, float* nu,
                         float* rl, float* ru, int64_t count, hipStream_t s)
{
    if (count <= 0) return;
    hipLaunchKernelGGL(relax_params_kernel, dim3((unsigned)ceil_div(count, kThreads)), dim3(kThreads), 0, s,
                       l, u, lambda, mu, nu, rl, ru, count);
    DPC_HIP(hipGetLastError());
}

void launch_relax_step(float* C, int ldc, double* cst, int nsides, int batch, int R, int n,
                       const float* lambda, const float* mu, const float* nu, const float* bias,
                       const float* shared_src, int ld_src, const float* cst_init, hipStream_t s)
{
    DPC_REQUIRE(C && cst && nsides >= 1 && nsides <= 2 && batch >= 0 && R >= 0 && n >= 1, DPC_EINVAL,
                "relax_step: bad arguments");
    DPC_REQUIRE(ldc >= n && ldc % 4 == 0 && ((uintptr_t)C % 16) == 0, DPC_EINVAL,
                "relax_step: ldc must be >= n and a multiple of 4, C 16-byte aligned");
    DPC_REQUIRE((lambda != nullptr) == (mu != nullptr) && (mu != nullptr) == (nu != nullptr), DPC_EINVAL,
                "relax_step: lambda, mu, nu must be given together");
    if (shared_src)
        DPC_REQUIRE(ld_src >= ldc && ld_src % 4 == 0 && ((uintptr_t)shared_src % 16) == 0, DPC_EINVAL,
                    "relax_step: shared source needs ld_src >= ldc, multiple of 4, 16-byte aligned");
    DPC_REQUIRE((int64_t)nsides * batch <= 65535, DPC_EINVAL, "relax_step: nsides*batch exceeds 65535");
    if (batch == 0 || R == 0) return;
    if (ldc <= 2048 && tune(TK_ROWS_STREAM)) {
        // parameters of a whole row in LDS (32 KB at most, so that five workgroups fit a compute unit): the streaming kernel
        const size_t lds_s = (size_t)ldc * 16;
        const int rpb = pick_rows_per_block(R, nsides * batch, (int)ceil_div(ldc, 1024));
        dim3 grid_s((unsigned)ceil_div(R, rpb), (unsigned)(nsides * batch));
        auto go = [&](auto kern) {
            if (lds_s > 48 * 1024) ensure_dynamic_lds((const void*)kern, 64 * 1024);
            hipLaunchKernelGGL(kern, grid_s, dim3(kThreads), lds_s, s, C, ldc, cst, batch, R, n, lambda, mu, nu, bias,
                               shared_src, shared_src ? ld_src : 0, cst_init, rpb);
        };
        // rows larger than the Infinity Cache stream past the caches
        const bool nt = (int64_t)nsides * batch * R * ldc * 4 > ((int64_t)384 << 20);
        if (shared_src) { if (nt) go(relax_step_stream_kernel<true, true>); else go(relax_step_stream_kernel<true, false>); }
        else { if (nt) go(relax_step_stream_kernel<false, true>); else go(relax_step_stream_kernel<false, false>); }
        DPC_HIP(hipGetLastError());
        return;
    }
    const int rpw = pick_rows_per_wave(R, nsides * batch);
    const int chunk = std::min(ldc, kChunk);
    const size_t lds = (size_t)chunk * 16;
    dim3 grid((unsigned)ceil_div(R, rpw * kWaves), (unsigned)(nsides * batch));
    if (shared_src)
        hipLaunchKernelGGL(relax_step_kernel<true>, grid, dim3(kThreads), lds, s, C, ldc, cst, batch, R, n,
                           lambda, mu, nu, bias, shared_src, ld_src, cst_init, rpw, chunk);
    else
        hipLaunchKernelGGL(relax_step_kernel<false>, grid, dim3(kThreads), lds, s, C, ldc, cst, batch, R, n,
                           lambda, mu, nu, bias, (const float*)nullptr, 0, cst_init, rpw, chunk);
    DPC_HIP(hipGetLastError());
}

void launch_concretise(const float* C, int ldc, const double* cst, int nsides, int batch, int R, int n,
                       const float* lo, const float* hi, float* out_l, float* out_u,
                       const float* shared_src, int ld_src, const float* cst_init, hipStream_t s,
                       const float* part, int nslots, int64_t part_stride)
{
    DPC_REQUIRE(nsides >= 1 && nsides <= 2 && batch >= 0 && R >= 0 && n >= 1 && lo && hi && out_l, DPC_EINVAL,
                "concretise: bad arguments");
    DPC_REQUIRE(nslots == 0 || (part && part_stride >= (int64_t)nsides * batch * R), DPC_EINVAL,
                "concretise: bad partial-sum slots");
    DPC_REQUIRE(nsides == 1 || out_u, DPC_EINVAL, "concretise: out_u missing");
    DPC_REQUIRE(ldc >= n && ldc % 4 == 0, DPC_EINVAL, "concretise: ldc must be >= n and a multiple of 4");
    if (shared_src)
        DPC_REQUIRE(ld_src >= ldc && ld_src % 4 == 0 && ((uintptr_t)shared_src % 16) == 0 && cst_init, DPC_EINVAL,
                    "concretise: shared source needs ld_src >= ldc, multiple of 4, 16-byte aligned, cst_init");
    else
        DPC_REQUIRE(C && cst && ((uintptr_t)C % 16) == 0, DPC_EINVAL, "concretise: C/cst missing or misaligned");
    DPC_REQUIRE((int64_t)nsides * batch <= 65535, DPC_EINVAL, "concretise: nsides*batch exceeds 65535");
    if (batch == 0 || R == 0) return;
    if (ldc <= 2048 && tune(TK_ROWS_STREAM)) {
        const size_t lds_s = (size_t)ldc * 8;
        const int rpb = pick_rows_per_block(R, nsides * batch, (int)ceil_div(ldc, 1024));
        dim3 grid_s((unsigned)ceil_div(R, rpb), (unsigned)(nsides * batch));
        auto go = [&](auto kern) {
            if (lds_s > 48 * 1024) ensure_dynamic_lds((const void*)kern, 64 * 1024);
            hipLaunchKernelGGL(kern, grid_s, dim3(kThreads), lds_s, s, C, ldc, cst, batch, R, n, lo, hi, out_l, out_u,
                               shared_src, shared_src ? ld_src : 0, cst_init, rpb, part, nslots, (long long)part_stride);
        };
        if (shared_src) go(concretise_stream_kernel<true>);
        else go(concretise_stream_kernel<false>);
        DPC_HIP(hipGetLastError());
        return;
    }
    const int rpw = pick_rows_per_wave(R, nsides * batch);
    const int chunk = std::min(ldc, kChunk);
    const size_t lds = (size_t)chunk * 8;
    dim3 grid((unsigned)ceil_div(R, rpw * kWaves), (unsigned)(nsides * batch));
    if (shared_src)
        hipLaunchKernelGGL(concretise_kernel<true>, grid, dim3(kThreads), lds, s, C, ldc, cst, batch, R, n, lo, hi,
                           out_l, out_u, shared_src, ld_src, cst_init, rpw, chunk, part, nslots, (long long)part_stride);
    else
        hipLaunchKernelGGL(concretise_kernel<false>, grid, dim3(kThreads), lds, s, C, ldc, cst, batch, R, n, lo, hi,
                           out_l, out_u, (const float*)nullptr, 0, cst_init, rpw, chunk, part, nslots,
                           (long long)part_stride);
    DPC_HIP(hipGetLastError());
}

void launch_pack_relax(const float* lambda, const float* mu, const float* nu, const float* bias, int batch, int n,
                       int ld, float* pk, hipStream_t s)
{
    DPC_REQUIRE(lambda && mu && nu && pk && ld >= n && ((uintptr_t)pk % 16) == 0, DPC_EINVAL, "pack_relax: bad arguments");
    const int64_t tot = (int64_t)2 * batch * ld;
    if (tot == 0) return;
    hipLaunchKernelGGL(pack_relax_kernel, dim3((unsigned)ceil_div(tot, kThreads)), dim3(kThreads), 0, s, lambda, mu, nu,
                       bias, batch, n, ld, reinterpret_cast<float4*>(pk));
    DPC_HIP(hipGetLastError());
}

void launch_merge_block(float* dst, int ld_dst, int64_t M, int R, int rows_C, int ph2, int pw2, int C, int kind,
                        const float* src, int ld_src, int ph1, int pw1, int d, hipStream_t s)
{
    DPC_REQUIRE(dst && M >= 0 && R >= 1 && rows_C >= 1 && C >= 1 && kind >= 0 && kind <= 2 && d >= 0, DPC_EINVAL,
                "merge_block: bad arguments");
    DPC_REQUIRE(ph1 >= 1 && pw1 >= 1 && ph1 + d <= ph2 && pw1 + d <= pw2 && (int64_t)ph2 * pw2 * C <= ld_dst, DPC_EINVAL,
                "merge_block: the waiting block does not fit the rows");
    DPC_REQUIRE(kind == 2 ? (ph1 == 1 && pw1 == 1 && rows_C <= C) : (src && (int64_t)ph1 * pw1 * C <= ld_src), DPC_EINVAL,
                "merge_block: bad source block");
    DPC_REQUIRE(M <= 0x7fffffff, DPC_EINVAL, "merge_block: too many rows");
    if (M == 0) return;
    MergeArgs a{dst, ld_dst, src, ld_src, R, rows_C, ph1, pw1, pw2, C, d, kind};
    hipLaunchKernelGGL(merge_block_kernel, dim3((unsigned)M), dim3(kThreads), 0, s, a);
    DPC_HIP(hipGetLastError());
}

void launch_block_bound(double* cst, int64_t M, int R, int rows_C, int rows_W, int batch, int nsides, int n, int kind,
                        const float* src, int ld_src, const float* lo, const float* hi, int patch, int ph, int pw, int C, int S,
                        int P, int gh, int gw, hipStream_t s)
{
    DPC_REQUIRE(cst && lo && hi && M >= 0 && R >= 1 && rows_C >= 1 && rows_W >= 1 && batch >= 1 && (nsides == 1 || nsides == 2) &&
                    n >= 1 && kind >= 0 && kind <= 2 && M == (int64_t)nsides * batch * R, DPC_EINVAL, "block_bound: bad arguments");
    DPC_REQUIRE(kind == 2 ? R <= n : (src && (patch ? (int64_t)ph * pw * C <= ld_src && (int64_t)gh * gw * C <= n : n <= ld_src)), DPC_EINVAL,
                "block_bound: the block does not fit its layer");
    if (M == 0) return;
    BlockBoundArgs a{cst, src, ld_src, lo, hi, (long long)M, R, rows_C, rows_W, batch, nsides, n, patch, ph, pw, C, S, P, gh, gw, kind};
    hipLaunchKernelGGL(block_bound_kernel, dim3((unsigned)ceil_div(M, kThreads / 64)), dim3(kThreads), 0, s, a);
    DPC_HIP(hipGetLastError());
}

// Patch-form rows that have reached the input layer written out as dense rows over it (kept symbolic bounds of a
// convolution layer's neurons): row m's ph x pw x C patch sits at grid position (ho*S - P, wo*S - P) of the gh x gw grid;
// positions off the grid carry no neuron.  shared_mod > 0: the rows are still the layer's own kernel cores,
// src row = (m % R) % shared_mod, constant = cst_init_c of that channel; else constants are copied.  dst is zero before.
struct ExpandArgs {
    const float* src; int ld_src; int shared_mod;
    const double* cst_in; const float* cst_init_c;
    float* dst; int ld_dst; double* cst_out;
    int R, rows_C, rows_W, ph, pw, C, S, P, gh, gw;
};

__global__ __launch_bounds__(kThreads) void expand_patch_rows_kernel(ExpandArgs a)
{
    const size_t m = blockIdx.x;
    const int r = (int)(m % (size_t)a.R);
    const size_t srow = a.shared_mod > 0 ? (size_t)(r % a.shared_mod) : m;
    const float* src = a.src + srow * a.ld_src;
    float* dst = a.dst + m * a.ld_dst;
    const int wo = (r / a.rows_C) % a.rows_W, ho = r / (a.rows_C * a.rows_W);
    const int oy = ho * a.S - a.P, ox = wo * a.S - a.P;
    const int n1 = a.ph * a.pw * a.C;
    for (int e = threadIdx.x; e < n1; e += kThreads) {
        const int pos = e / a.C, c = e - pos * a.C;
        const int py = pos / a.pw, px = pos - py * a.pw;
        const int gy = oy + py, gx = ox + px;
        if (gy < 0 || gy >= a.gh || gx < 0 || gx >= a.gw) continue;
        dst[(size_t)(gy * a.gw + gx) * a.C + c] = src[e];
    }
    if (threadIdx.x == 0) a.cst_out[m] = a.shared_mod > 0 ? (double)a.cst_init_c[r % a.shared_mod] : a.cst_in[m];
}

void launch_expand_patch_rows(const float* src, int ld_src, int shared_mod, const double* cst_in, const float* cst_init_c,
                              int64_t M, int R, int rows_C, int rows_W, int ph, int pw, int C, int S, int P, int gh, int gw,
                              float* dst, int ld_dst, double* cst_out, hipStream_t s)
{
    DPC_REQUIRE(src && dst && cst_out && M >= 0 && M <= 0x7fffffff && R >= 1 && rows_C >= 1 && rows_W >= 1 && ph >= 1 && pw >= 1 && C >= 1 &&
                    S >= 1 && P >= 0 && gh >= 1 && gw >= 1, DPC_EINVAL, "expand_patch_rows: bad arguments");
    DPC_REQUIRE((int64_t)ph * pw * C <= ld_src && (int64_t)gh * gw * C <= ld_dst, DPC_EINVAL, "expand_patch_rows: rows do not fit");
    DPC_REQUIRE(shared_mod > 0 ? cst_init_c != nullptr : cst_in != nullptr, DPC_EINVAL, "expand_patch_rows: no constants");
    if (M == 0) return;
    ExpandArgs a{src, ld_src, shared_mod, cst_in, cst_init_c, dst, ld_dst, cst_out, R, rows_C, rows_W, ph, pw, C, S, P, gh, gw};
    hipLaunchKernelGGL(expand_patch_rows_kernel, dim3((unsigned)M), dim3(kThreads), 0, s, a);
    DPC_HIP(hipGetLastError());
}

// Kept symbolic bounds of one input, from the internal neuron orders to the interface's: out[r'][j'] = src[r][j] with
// r' / j' the (C,H,W) positions of the (H,W,C)-ordered row r / column j (rC or cC = 0: that side has no shape);
// constants double -> float.
struct SymExportArgs {
    const float* src; int ld_src; const double* cst;
    float* out; float* cst_out;
    int n, n0, rC, rH, rW, cC, cH, cW;
};

__global__ __launch_bounds__(kThreads) void sym_export_kernel(SymExportArgs a)
{
    const int r = blockIdx.x;                      // internal row index
    int ro = r;
    if (a.rC > 0) {
        const int c = r % a.rC, pos = r / a.rC;
        ro = c * a.rH * a.rW + pos;
    }
    if (a.out) {
        const float* src = a.src + (size_t)r * a.ld_src;
        float* out = a.out + (size_t)ro * a.n0;
        for (int j = threadIdx.x; j < a.n0; j += kThreads) {
            int jo = j;
            if (a.cC > 0) {
                const int c = j % a.cC, pos = j / a.cC;
                jo = c * a.cH * a.cW + pos;
            }
            out[jo] = src[j];
        }
    }
    if (a.cst_out && threadIdx.x == 0) a.cst_out[ro] = (float)a.cst[r];
}

void launch_sym_export(const float* src, int ld_src, const double* cst, int n, int n0, int rC, int rH, int rW, int cC, int cH, int cW,
                       float* out, float* cst_out, hipStream_t s)
{
    DPC_REQUIRE(src && cst && n >= 1 && n0 >= 1 && n0 <= ld_src, DPC_EINVAL, "sym_export: bad arguments");
    DPC_REQUIRE((rC == 0 || (int64_t)rC * rH * rW == n) && (cC == 0 || (int64_t)cC * cH * cW == n0), DPC_EINVAL, "sym_export: shapes do not match sizes");
    SymExportArgs a{src, ld_src, cst, out, cst_out, n, n0, rC, rH, rW, cC, cH, cW};
    hipLaunchKernelGGL(sym_export_kernel, dim3((unsigned)n), dim3(kThreads), 0, s, a);
    DPC_HIP(hipGetLastError());
}

// rows[r][0:ncols] *= scale[r];  cst[r] = scale[r] * (bias_f ? bias_f[r] : cst[r]) + (add ? add[r] : 0): a ReLU neuron's
// polyhedral bound written over the neurons two layers back (scale = lambda or mu, add = nu) from the rows of the
// layer under it.
__global__ __launch_bounds__(kThreads) void scale_rows_kernel(float* __restrict__ rows, int ld, int ncols, double* __restrict__ cst,
                                                              const float* __restrict__ bias_f, const float* __restrict__ scale,
                                                              const float* __restrict__ add)
{
    const int r = blockIdx.x;
    const float sc = scale[r];
    float* row = rows + (size_t)r * ld;
    for (int j = threadIdx.x; j < ncols; j += kThreads) row[j] *= sc;
    if (threadIdx.x == 0) cst[r] = (double)sc * (bias_f ? (double)bias_f[r] : cst[r]) + (add ? (double)add[r] : 0.0);
}

void launch_scale_rows(float* rows, int ld, int n, int ncols, double* cst, const float* bias_f, const float* scale, const float* add,
                       hipStream_t s)
{
    DPC_REQUIRE(rows && cst && scale && n >= 1 && ncols >= 1 && ncols <= ld, DPC_EINVAL, "scale_rows: bad arguments");
    hipLaunchKernelGGL(scale_rows_kernel, dim3((unsigned)n), dim3(kThreads), 0, s, rows, ld, ncols, cst, bias_f, scale, add);
    DPC_HIP(hipGetLastError());
}

__global__ __launch_bounds__(kThreads) void fill_zero_kernel(float* __restrict__ p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}

void launch_fill_zero(float* p, int64_t n, hipStream_t s)
{
    DPC_REQUIRE(p && n >= 0 && ceil_div(n, kThreads) < ((int64_t)1 << 31), DPC_EINVAL, "fill_zero: bad arguments");
    if (n == 0) return;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)ceil_div(n, kThreads)), dim3(kThreads), 0, s, p, n);
    DPC_HIP(hipGetLastError());
}

// cst[m] += sum over k < nslots of part[k * stride + m], in index order
// (init given: cst[m] = init[m % init_mod] + that sum, the rows' first constants)
__global__ __launch_bounds__(kThreads) void fold_slots_kernel(double* __restrict__ cst, const float* __restrict__ part, int nslots,
                                                              long long stride, int64_t M, const float* __restrict__ init, int init_mod)
{
    const int64_t m = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (m >= M) return;
    double t = 0.0;
    for (int k = 0; k < nslots; ++k) t += (double)part[(size_t)k * stride + m];
    cst[m] = (init ? (double)init[m % init_mod] : cst[m]) + t;
}

void launch_fold_slots(double* cst, const float* part, int nslots, int64_t stride, int64_t M, hipStream_t s, const float* init, int init_mod)
{
    DPC_REQUIRE(cst && part && nslots >= 0 && stride >= M && M >= 0 && (!init || init_mod > 0), DPC_EINVAL, "fold_slots: bad arguments");
    if (M == 0 || (nslots == 0 && !init)) return;
    hipLaunchKernelGGL(fold_slots_kernel, dim3((unsigned)ceil_div(M, kThreads)), dim3(kThreads), 0, s, cst, part, nslots, (long long)stride, M,
                       init, init_mod);
    DPC_HIP(hipGetLastError());
}

// out[i] = a[i] + b[i]
__global__ __launch_bounds__(kThreads) void add_vectors_kernel(const float* __restrict__ a, const float* __restrict__ b,
                                                               float* __restrict__ out, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) out[i] = a[i] + b[i];
}

void launch_add_vectors(const float* a, const float* b, float* out, int64_t n, hipStream_t s)
{
    DPC_REQUIRE(a && b && out && n >= 0, DPC_EINVAL, "add_vectors: bad arguments");
    if (n == 0) return;
    hipLaunchKernelGGL(add_vectors_kernel, dim3((unsigned)ceil_div(n, kThreads)), dim3(kThreads), 0, s, a, b, out, n);
    DPC_HIP(hipGetLastError());
}

void launch_pack_relax2(const float* lambda, const float* mu, const float* nu, int batch, int n, int ld, float* pk2,
                        hipStream_t s)
{
    DPC_REQUIRE(lambda && mu && nu && pk2 && ld >= n && ((uintptr_t)pk2 % 16) == 0, DPC_EINVAL, "pack_relax2: bad arguments");
    const int64_t tot = (int64_t)batch * ld;
    if (tot == 0) return;
    hipLaunchKernelGGL(pack_relax2_kernel, dim3((unsigned)ceil_div(tot, kThreads)), dim3(kThreads), 0, s, lambda, mu, nu, batch,
                       n, ld, reinterpret_cast<float2*>(pk2));
    DPC_HIP(hipGetLastError());
}

void launch_pack_bounds(const float* lo, const float* hi, int batch, int n, int ld, float* pk, hipStream_t s)
{
    DPC_REQUIRE(lo && hi && pk && ld >= n && ((uintptr_t)pk % 16) == 0, DPC_EINVAL, "pack_bounds: bad arguments");
    const int64_t tot = (int64_t)2 * batch * ld;
    if (tot == 0) return;
    hipLaunchKernelGGL(pack_bounds_kernel, dim3((unsigned)ceil_div(tot, kThreads)), dim3(kThreads), 0, s, lo, hi, batch, n,
                       ld, reinterpret_cast<float4*>(pk));
    DPC_HIP(hipGetLastError());
}

void launch_finalize_bounds(const double* cst, const float* part, int nslots, int64_t part_stride, int nsides, int batch,
                            int R, float* out_l, float* out_u, hipStream_t s)
{
    const int64_t M = (int64_t)nsides * batch * R;
    DPC_REQUIRE(cst && out_l && (nsides == 1 || out_u) && (nslots == 0 || (part && part_stride >= M)), DPC_EINVAL,
                "finalize_bounds: bad arguments");
    if (M == 0) return;
    hipLaunchKernelGGL(finalize_bounds_kernel, dim3((unsigned)ceil_div(M, kThreads)), dim3(kThreads), 0, s, cst, part, nslots,
                       (long long)part_stride, batch, R, (long long)M, out_l, out_u);
    DPC_HIP(hipGetLastError());
}

void launch_finalize_relax_pack(const double* cst, const float* part, int nslots, int64_t part_stride, float* out_l, float* out_u,
                                float* lambda, float* mu, float* nu, float* rl, float* ru, const float* bias, int batch, int n, int ld,
                                float* pk, float* pk2, hipStream_t s)
{
    DPC_REQUIRE(cst && out_l && out_u && lambda && mu && nu && rl && ru && ld >= n && ((uintptr_t)pk % 16) == 0 && ((uintptr_t)pk2 % 8) == 0 &&
                    (nslots == 0 || (part && part_stride >= (int64_t)2 * batch * n)), DPC_EINVAL, "finalize_relax_pack: bad arguments");
    const int64_t tot = (int64_t)batch * ld;
    if (tot <= 0) return;
    hipLaunchKernelGGL(finalize_relax_pack_kernel, dim3((unsigned)ceil_div(tot, kThreads)), dim3(kThreads), 0, s, cst, part, nslots,
                       (long long)part_stride, out_l, out_u, lambda, mu, nu, rl, ru, bias, batch, n, ld, reinterpret_cast<float4*>(pk),
                       reinterpret_cast<float2*>(pk2));
    DPC_HIP(hipGetLastError());
}

bool launch_finalize_split_final(const double* cst, const float* part, int nslots, int64_t part_stride, int batch, int nK, int Rs, float* l,
                                 float* u, float* margin, int32_t* verdict, hipStream_t s)
{
    if (Rs > 64 || Rs < 2 * nK - 1 || nK < 2) return false;
    DPC_REQUIRE(cst && l && u && margin && verdict && (nslots == 0 || (part && part_stride >= (int64_t)2 * batch * Rs)), DPC_EINVAL,
                "finalize_split_final: bad arguments");
    if (batch == 0) return true;
    hipLaunchKernelGGL(finalize_split_final_kernel, dim3((unsigned)batch), dim3(64), 0, s, cst, part, nslots, (long long)part_stride, batch,
                       nK, Rs, l, u, margin, verdict);
    DPC_HIP(hipGetLastError());
    return true;
}

void launch_margin_rows(const float* W, int ldw, const float* bias, const int32_t* label, int batch,
                        int nK, int n, float* C, int ldc, double* cst, hipStream_t s)
{
    DPC_REQUIRE(nK >= 2 && ldc >= n && ldw >= n, DPC_EINVAL, "margin_rows: bad shape");
    if (batch == 0) return;
    hipLaunchKernelGGL(margin_rows_kernel, dim3((unsigned)(batch * (nK - 1))), dim3(kThreads), 0, s,
                       W, ldw, bias, label, nK, n, C, ldc, cst);
    DPC_HIP(hipGetLastError());
}

void launch_final_rows(const float* W, int ldw, const float* bias, const int32_t* label, int batch, int nK, int n,
                       float* C, int ldc, double* cst, hipStream_t s, int Rs)
{
    if (Rs <= 0) Rs = 2 * nK - 1;
    DPC_REQUIRE(nK >= 2 && ldc >= n && ldw >= n && Rs >= 2 * nK - 1, DPC_EINVAL, "final_rows: bad shape");
    if (batch == 0) return;
    hipLaunchKernelGGL(final_rows_kernel, dim3((unsigned)(2 * batch * Rs)), dim3(kThreads), 0, s, W, ldw, bias,
                       label, batch, nK, n, C, ldc, cst, Rs);
    DPC_HIP(hipGetLastError());
}

void launch_split_final(const float* tl, const float* tu, int batch, int nK, float* l, float* u, float* margin,
                        int32_t* verdict, hipStream_t s, int Rs)
{
    if (batch == 0) return;
    if (Rs <= 0) Rs = 2 * nK - 1;
    hipLaunchKernelGGL(split_final_kernel, dim3((unsigned)ceil_div(batch, 64)), dim3(64), 0, s, tl, tu, batch, nK, l, u,
                       margin, verdict, Rs);
    DPC_HIP(hipGetLastError());
}

void launch_verdict(const float* margin, int batch, int nq, int32_t* verdict, hipStream_t s)
{
    if (batch == 0) return;
    hipLaunchKernelGGL(verdict_kernel, dim3((unsigned)ceil_div(batch, 64)), dim3(64), 0, s, margin, batch, nq, verdict);
    DPC_HIP(hipGetLastError());
}

void launch_chw_to_hwc(const float* src, float* dst, int batch, int C, int H, int W, hipStream_t s)
{
    const int64_t tot = (int64_t)batch * C * H * W;
    if (tot == 0) return;
    hipLaunchKernelGGL(permute_kernel<true>, dim3((unsigned)ceil_div(tot, kThreads)), dim3(kThreads), 0, s,
                       src, dst, batch, C, H, W);
    DPC_HIP(hipGetLastError());
}

void launch_hwc_to_chw(const float* src, float* dst, int batch, int C, int H, int W, hipStream_t s)
{
    const int64_t tot = (int64_t)batch * C * H * W;
    if (tot == 0) return;
    hipLaunchKernelGGL(permute_kernel<false>, dim3((unsigned)ceil_div(tot, kThreads)), dim3(kThreads), 0, s,
                       src, dst, batch, C, H, W);
    DPC_HIP(hipGetLastError());
}

}  // namespace dpc
