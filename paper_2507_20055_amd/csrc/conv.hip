// Convolution-layer kernels of the back-substitution (patch-form rows, transposed convolution)
// and input validation.
#include <vector>

#include "conv.h"

namespace dpc {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

struct PatchArgs {
    int rows_W, rows_C, ph, pw, C, S, P, gh, gw, elems;
};

// One wavefront per row; lanes stride over the patch elements (channel fastest, so a wavefront
// reads contiguous runs of the row and contiguous channel vectors of the per-input parameters).
template <bool SHARED>
__global__ __launch_bounds__(kThreads) void relax_step_patch_kernel(
    float* __restrict__ C, int ldc, double* __restrict__ cst, int batch, int R, PatchArgs pa,
    const float* __restrict__ lambda, const float* __restrict__ mu, const float* __restrict__ nu,
    const float* __restrict__ bias_c, const float* __restrict__ core, int ld_core,
    const float* __restrict__ cst_init_c, int rows_per_wave)
{
    const int sb = blockIdx.y;
    const int side = sb / batch, b = sb - side * batch;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r0 = (blockIdx.x * kWaves + wave) * rows_per_wave;
    const size_t pbase = (size_t)b * pa.gh * pa.gw * pa.C;
    for (int q = 0; q < rows_per_wave; ++q) {
        const int r = r0 + q;
        if (r >= R) break;
        const int co = r % pa.rows_C, wo = (r / pa.rows_C) % pa.rows_W, ho = r / (pa.rows_C * pa.rows_W);
        const int oy = ho * pa.S - pa.P, ox = wo * pa.S - pa.P;
        const size_t m = (size_t)sb * R + r;
        const float* in = SHARED ? core + (size_t)co * ld_core : C + m * ldc;
        float* out = C + m * ldc;
        double a = 0.0;
        for (int e = lane; e < ldc; e += 64) {
            float y = 0.0f;
            if (e < pa.elems) {
                const int c = e % pa.C, pos = e / pa.C;
                const int px = pos % pa.pw, py = pos / pa.pw;
                const int gy = oy + py, gx = ox + px;
                if (gy >= 0 && gy < pa.gh && gx >= 0 && gx < pa.gw) {
                    const size_t idx = pbase + ((size_t)gy * pa.gw + gx) * pa.C + c;
                    const float la = lambda ? lambda[idx] : 1.0f;
                    const float mm = mu ? mu[idx] : 1.0f;
                    const float v = nu ? nu[idx] : 0.0f;
                    const float bj = bias_c ? bias_c[c] : 0.0f;
                    const float x = in[e];
                    const bool pos_c = x >= 0.0f;
                    const float mult = pos_c ? (side == 0 ? la : mm) : (side == 0 ? mm : la);
                    const float k = ((pos_c == (side != 0)) ? v : 0.0f) + mult * bj;
                    y = x * mult;
                    a += (double)x * (double)k;
                }
            }
            out[e] = y;
        }
        const double t = wave_sum(a);
        if (lane == 0) cst[m] = (SHARED ? (double)cst_init_c[co] : cst[m]) + t;
    }
}

template <bool SHARED>
__global__ __launch_bounds__(kThreads) void concretise_patch_kernel(
    const float* __restrict__ C, int ldc, const double* __restrict__ cst, int batch, int R, PatchArgs pa,
    const float* __restrict__ lo, const float* __restrict__ hi, float* __restrict__ out_l, float* __restrict__ out_u,
    const float* __restrict__ core, int ld_core, const float* __restrict__ cst_init_c, int rows_per_wave)
{
    const int sb = blockIdx.y;
    const int side = sb / batch, b = sb - side * batch;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r0 = (blockIdx.x * kWaves + wave) * rows_per_wave;
    const size_t pbase = (size_t)b * pa.gh * pa.gw * pa.C;
    for (int q = 0; q < rows_per_wave; ++q) {
        const int r = r0 + q;
        if (r >= R) break;
        const int co = r % pa.rows_C, wo = (r / pa.rows_C) % pa.rows_W, ho = r / (pa.rows_C * pa.rows_W);
        const int oy = ho * pa.S - pa.P, ox = wo * pa.S - pa.P;
        const size_t m = (size_t)sb * R + r;
        const float* in = SHARED ? core + (size_t)co * ld_core : C + m * ldc;
        double a = 0.0;
        for (int e = lane; e < pa.elems; e += 64) {
            const int c = e % pa.C, pos = e / pa.C;
            const int px = pos % pa.pw, py = pos / pa.pw;
            const int gy = oy + py, gx = ox + px;
            if (gy >= 0 && gy < pa.gh && gx >= 0 && gx < pa.gw) {
                const size_t idx = pbase + ((size_t)gy * pa.gw + gx) * pa.C + c;
                const float x = in[e];
                const float bound = (x >= 0.0f) == (side == 0) ? lo[idx] : hi[idx];
                a += (double)x * (double)bound;
            }
        }
        const double t = wave_sum(a);
        if (lane == 0) {
            const double v = (SHARED ? (double)cst_init_c[co] : cst[m]) + t;
            (side == 0 ? out_l : out_u)[(size_t)b * R + r] = (float)v;
        }
    }
}

// Shared small cores (a convolution layer's own kernel as the expressions of its neurons: interval bounds of the first
// layer): one THREAD per row.  The cores sit in LDS, the lanes of a wavefront are consecutive channels of a few
// positions, so the box values they read are broadcasts; a row's products are added in element order in fp64.
__global__ __launch_bounds__(kThreads) void concretise_patch_small_kernel(
    int batch, int R, PatchArgs pa, const float* __restrict__ lo, const float* __restrict__ hi, float* __restrict__ out_l,
    float* __restrict__ out_u, const float* __restrict__ core, int ld_core, const float* __restrict__ cst_init_c)
{
    extern __shared__ float s_core[];                  // [rows_C][elems + 1]
    const int es = pa.elems + 1;
    for (int i = threadIdx.x; i < pa.rows_C * pa.elems; i += kThreads) {
        const int co = i / pa.elems, e = i - co * pa.elems;
        s_core[co * es + e] = core[(size_t)co * ld_core + e];
    }
    __syncthreads();
    const int sb = blockIdx.y;
    const int side = sb / batch, b = sb - side * batch;
    const int r = blockIdx.x * kThreads + threadIdx.x;
    if (r >= R) return;
    const int co = r % pa.rows_C, wo = (r / pa.rows_C) % pa.rows_W, ho = r / (pa.rows_C * pa.rows_W);
    const int oy = ho * pa.S - pa.P, ox = wo * pa.S - pa.P;
    const size_t pbase = (size_t)b * pa.gh * pa.gw * pa.C;
    const float* in = s_core + co * es;
    double a = 0.0;
    for (int py = 0; py < pa.ph; ++py) {
        const int gy = oy + py;
        if (gy < 0 || gy >= pa.gh) continue;
        for (int px = 0; px < pa.pw; ++px) {
            const int gx = ox + px;
            if (gx < 0 || gx >= pa.gw) continue;
            const size_t idx = pbase + ((size_t)gy * pa.gw + gx) * pa.C;
            const float* x = in + (py * pa.pw + px) * pa.C;
            for (int c = 0; c < pa.C; ++c) {
                const float bound = (x[c] >= 0.0f) == (side == 0) ? lo[idx + c] : hi[idx + c];
                a += (double)x[c] * (double)bound;
            }
        }
    }
    (side == 0 ? out_l : out_u)[(size_t)b * R + r] = (float)((double)cst_init_c[co] + a);
}

// Transposed convolution of coefficient rows, one thread per output element (gather form: every
// output is produced by exactly one thread, so the summation order is fixed).
__global__ __launch_bounds__(kThreads) void conv_transpose_rows_kernel(
    const float* __restrict__ in, int ld_in, int ih, int iw, int Co, int Ci, int kh, int kw, int stride,
    const float* __restrict__ taps, float* __restrict__ out, int ld_out, int oh, int ow, int off)
{
    const size_t m = blockIdx.x;
    const int o = blockIdx.y * kThreads + threadIdx.x;
    if (o >= ld_out) return;
    float acc = 0.0f;
    if (o < oh * ow * Ci) {
        const int ci = o % Ci, x = (o / Ci) % ow, y = o / (Ci * ow);
        const float* row = in + m * ld_in;
        for (int ky = 0; ky < kh; ++ky) {
            const int ty = y + off - ky;
            if (ty < 0 || ty % stride != 0) continue;
            const int py = ty / stride;
            if (py >= ih) continue;
            for (int kx = 0; kx < kw; ++kx) {
                const int tx = x + off - kx;
                if (tx < 0 || tx % stride != 0) continue;
                const int px = tx / stride;
                if (px >= iw) continue;
                const float* p = row + ((size_t)py * iw + px) * Co;
                const float* t = taps + ((size_t)(ky * kw + kx) * Co) * Ci + ci;
                for (int co = 0; co < Co; ++co) acc = fmaf(p[co], t[(size_t)co * Ci], acc);
            }
        }
    }
    out[m * ld_out + o] = acc;
}

__global__ void check_inputs_kernel(const float* __restrict__ lo, const float* __restrict__ hi, size_t count,
                                    const int32_t* __restrict__ label, int batch, int nK, int32_t* __restrict__ flag)
{
    int bad = 0;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x) {
        const float a = lo[i], b = hi[i];
        if (!(a <= b) || !isfinite(a) || !isfinite(b)) bad |= 1;
    }
    if (label)
        for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < (size_t)batch; i += (size_t)gridDim.x * blockDim.x)
            if (label[i] < 0 || label[i] >= nK) bad |= 2;
    if (bad) atomicOr(flag, bad);
}

// Boxes and labels that already live in device memory: copied into the result's buffers (spatial inputs go from the
// caller's (C,H,W) order to the internal (H,W,C) order) and validated in the same pass.  The flag word must be zero
// when the kernel starts.
__global__ void ingest_kernel(const float* __restrict__ lo, const float* __restrict__ hi, const int32_t* __restrict__ label,
                              float* __restrict__ l0, float* __restrict__ u0, int32_t* __restrict__ lab, int batch, int n0,
                              int Cc, int H, int W, int nK, int32_t* __restrict__ flag, float4* __restrict__ pk, int ld)
{
    // one destination element per step: (input, column of the internal order); with pk the box is also written in the
    // packed form of launch_pack_bounds ([side][input][ld] of (0, 0, bound the side takes under a coefficient >= 0, the
    // other bound), padding columns zero), which then needs no launch of its own
    int bad = 0;
    const size_t count = (size_t)batch * ld;
    for (size_t j = (size_t)blockIdx.x * blockDim.x + threadIdx.x; j < count; j += (size_t)gridDim.x * blockDim.x) {
        const size_t bi = j / ld;
        const int col = (int)(j - bi * ld);
        float4 lo4 = make_float4(0.f, 0.f, 0.f, 0.f), up4 = lo4;
        if (col < n0) {
            size_t si = bi * n0 + col;
            if (Cc > 0) {
                const int c = col % Cc, hw = col / Cc;
                const int w = hw % W, h = hw / W;
                si = bi * n0 + ((size_t)c * H + h) * W + w;
            }
            const float a = lo[si], b = hi[si];
            if (!(a <= b) || !isfinite(a) || !isfinite(b)) bad |= 1;
            l0[bi * n0 + col] = a;
            u0[bi * n0 + col] = b;
            lo4.z = a; lo4.w = b;
            up4.z = b; up4.w = a;
        }
        if (pk) {
            pk[j] = lo4;
            pk[count + j] = up4;
        }
    }
    if (label)
        for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < (size_t)batch; i += (size_t)gridDim.x * blockDim.x) {
            const int32_t v = label[i];
            lab[i] = v;
            if (v < 0 || v >= nK) bad |= 2;
        }
    if (bad) atomicOr(flag, bad);
}

__global__ void zero_word_kernel(int32_t* p) { *p = 0; }

PatchArgs to_args(const PatchGeom& g)
{
    return PatchArgs{g.rows_W, g.rows_C, g.ph, g.pw, g.C, g.S, g.P, g.gh, g.gw, g.elems()};
}

int rows_per_wave_for(int R, int groups)
{
    int rpw = 8;
    while (rpw > 1 && ceil_div(R, rpw * kWaves) * groups < 2048) rpw >>= 1;
    return rpw;
}

}  // namespace

ConvWeights::~ConvWeights()
{
    if (core) (void)hipFree(core);
    if (taps) (void)hipFree(taps);
    if (taps4) (void)hipFree(taps4);
    if (bias_c) (void)hipFree(bias_c);
}

void upload_conv_weights(const ConvGeom& g, const float* K, const float* b, ConvWeights& out)
{
    const int patch = g.kh * g.kw * g.Ci;
    out.ld_core = (int)round_up(patch, 4);
    std::vector<float> core((size_t)g.Co * out.ld_core, 0.0f), taps((size_t)g.kh * g.kw * g.Co * g.Ci);
    for (int co = 0; co < g.Co; ++co)
        for (int ci = 0; ci < g.Ci; ++ci)
            for (int ky = 0; ky < g.kh; ++ky)
                for (int kx = 0; kx < g.kw; ++kx) {
                    const float v = K[(((size_t)co * g.Ci + ci) * g.kh + ky) * g.kw + kx];
                    core[(size_t)co * out.ld_core + ((size_t)ky * g.kw + kx) * g.Ci + ci] = v;
                    taps[(((size_t)ky * g.kw + kx) * g.Co + co) * g.Ci + ci] = v;
                }
    DPC_HIP(hipMalloc(reinterpret_cast<void**>(&out.core), core.size() * sizeof(float)));
    DPC_HIP(hipMalloc(reinterpret_cast<void**>(&out.taps), taps.size() * sizeof(float)));
    DPC_HIP(hipMalloc(reinterpret_cast<void**>(&out.bias_c), (size_t)g.Co * sizeof(float)));
    DPC_HIP(hipMemcpy(out.core, core.data(), core.size() * sizeof(float), hipMemcpyHostToDevice));
    DPC_HIP(hipMemcpy(out.taps, taps.data(), taps.size() * sizeof(float), hipMemcpyHostToDevice));
    DPC_HIP(hipMemcpy(out.bias_c, b, (size_t)g.Co * sizeof(float), hipMemcpyHostToDevice));
    if (g.Co % 4 == 0) {
        std::vector<float> t4(taps.size());
        for (int t = 0; t < g.kh * g.kw; ++t)
            for (int co = 0; co < g.Co; ++co)
                for (int ci = 0; ci < g.Ci; ++ci)
                    t4[((((size_t)t * (g.Co / 4) + co / 4) * g.Ci + ci) << 2) + (co & 3)] = taps[((size_t)t * g.Co + co) * g.Ci + ci];
        DPC_HIP(hipMalloc(reinterpret_cast<void**>(&out.taps4), t4.size() * sizeof(float)));
        DPC_HIP(hipMemcpy(out.taps4, t4.data(), t4.size() * sizeof(float), hipMemcpyHostToDevice));
    }
}

void launch_relax_step_patch(float* C, int ldc, double* cst, int nsides, int batch, int R, const PatchGeom& pg,
                             const float* lambda, const float* mu, const float* nu, const float* bias_c,
                             const float* shared_core, int ld_core, const float* cst_init_c, hipStream_t s)
{
    DPC_REQUIRE(C && cst && nsides >= 1 && nsides <= 2 && batch >= 0 && R >= 0, DPC_EINVAL, "relax_step_patch: bad arguments");
    DPC_REQUIRE(ldc >= pg.elems() && R == R / (pg.rows_C * pg.rows_W) * (pg.rows_C * pg.rows_W), DPC_EINVAL,
                "relax_step_patch: row geometry does not match R");
    DPC_REQUIRE((lambda != nullptr) == (mu != nullptr) && (mu != nullptr) == (nu != nullptr), DPC_EINVAL,
                "relax_step_patch: lambda, mu, nu must be given together");
    if (shared_core) DPC_REQUIRE(ld_core >= pg.elems() && cst_init_c, DPC_EINVAL, "relax_step_patch: bad shared core");
    DPC_REQUIRE((int64_t)nsides * batch <= 65535, DPC_EINVAL, "relax_step_patch: nsides*batch exceeds 65535");
    if (batch == 0 || R == 0) return;
    const int rpw = rows_per_wave_for(R, nsides * batch);
    dim3 grid((unsigned)ceil_div(R, rpw * kWaves), (unsigned)(nsides * batch));
    if (shared_core)
        hipLaunchKernelGGL(relax_step_patch_kernel<true>, grid, dim3(kThreads), 0, s, C, ldc, cst, batch, R, to_args(pg),
                           lambda, mu, nu, bias_c, shared_core, ld_core, cst_init_c, rpw);
    else
        hipLaunchKernelGGL(relax_step_patch_kernel<false>, grid, dim3(kThreads), 0, s, C, ldc, cst, batch, R, to_args(pg),
                           lambda, mu, nu, bias_c, (const float*)nullptr, 0, (const float*)nullptr, rpw);
    DPC_HIP(hipGetLastError());
}

void launch_concretise_patch(const float* C, int ldc, const double* cst, int nsides, int batch, int R,
                             const PatchGeom& pg, const float* lo, const float* hi, float* out_l, float* out_u,
                             const float* shared_core, int ld_core, const float* cst_init_c, hipStream_t s)
{
    DPC_REQUIRE(nsides >= 1 && nsides <= 2 && batch >= 0 && R >= 0 && lo && hi && out_l && (nsides == 1 || out_u),
                DPC_EINVAL, "concretise_patch: bad arguments");
    DPC_REQUIRE(R == R / (pg.rows_C * pg.rows_W) * (pg.rows_C * pg.rows_W), DPC_EINVAL,
                "concretise_patch: row geometry does not match R");
    if (shared_core) DPC_REQUIRE(ld_core >= pg.elems() && cst_init_c, DPC_EINVAL, "concretise_patch: bad shared core");
    else DPC_REQUIRE(C && cst && ldc >= pg.elems(), DPC_EINVAL, "concretise_patch: bad rows");
    DPC_REQUIRE((int64_t)nsides * batch <= 65535, DPC_EINVAL, "concretise_patch: nsides*batch exceeds 65535");
    if (batch == 0 || R == 0) return;
    const int rpw = rows_per_wave_for(R, nsides * batch);
    dim3 grid((unsigned)ceil_div(R, rpw * kWaves), (unsigned)(nsides * batch));
    const size_t small_lds = (size_t)pg.rows_C * (pg.elems() + 1) * sizeof(float);
    if (shared_core && pg.elems() <= 256 && small_lds <= 32 * 1024) {
        dim3 g2((unsigned)ceil_div(R, kThreads), (unsigned)(nsides * batch));
        hipLaunchKernelGGL(concretise_patch_small_kernel, g2, dim3(kThreads), small_lds, s, batch, R, to_args(pg), lo, hi, out_l, out_u,
                           shared_core, ld_core, cst_init_c);
    } else if (shared_core)
        hipLaunchKernelGGL(concretise_patch_kernel<true>, grid, dim3(kThreads), 0, s, C, ldc, cst, batch, R, to_args(pg),
                           lo, hi, out_l, out_u, shared_core, ld_core, cst_init_c, rpw);
    else
        hipLaunchKernelGGL(concretise_patch_kernel<false>, grid, dim3(kThreads), 0, s, C, ldc, cst, batch, R, to_args(pg),
                           lo, hi, out_l, out_u, (const float*)nullptr, 0, (const float*)nullptr, rpw);
    DPC_HIP(hipGetLastError());
}

double launch_conv_transpose_rows(const float* in, int64_t M, int ld_in, int ih, int iw, const ConvGeom& g,
                                  const ConvWeights& w, float* out, int ld_out, int oh, int ow, int off, hipStream_t s)
{
    DPC_REQUIRE(in && out && M >= 0 && w.taps, DPC_EINVAL, "conv_transpose_rows: bad arguments");
    DPC_REQUIRE(ld_in >= ih * iw * g.Co && ld_out >= oh * ow * g.Ci, DPC_EINVAL,
                "conv_transpose_rows: leading dimensions too small");
    DPC_REQUIRE(M < ((int64_t)1 << 31), DPC_EINVAL, "conv_transpose_rows: too many rows");
    if (M == 0) return 0.0;
    const double flop = 2.0 * (double)M * ih * iw * g.Co * g.Ci * g.kh * g.kw;
    if (conv_algo() != 1 && launch_conv_transpose_fast(in, M, ld_in, ih, iw, g, w, out, ld_out, oh, ow, off, s)) return flop;
    dim3 grid((unsigned)M, (unsigned)ceil_div(ld_out, kThreads));
    hipLaunchKernelGGL(conv_transpose_rows_kernel, grid, dim3(kThreads), 0, s, in, ld_in, ih, iw, g.Co, g.Ci, g.kh, g.kw,
                       g.stride, w.taps, out, ld_out, oh, ow, off);
    DPC_HIP(hipGetLastError());
    return flop;
}

// 0: MFMA kernels where they apply; 1: always the generic gather kernel; 2: as 0, but few input channels go to the plain-ALU
// kernel instead of the MFMA one
int conv_algo() { return tune(TK_CONV_ALGO); }
// 1: 16 x 16 tiles in the MFMA kernel for layers with at most 16 input channels; 0: 32 x 32 always
int conv_half_tiles() { return tune(TK_CONV_HALF_TILES); }

int check_inputs(const float* lo, const float* hi, size_t count, const int32_t* label, int batch, int nK,
                 int32_t* flag, hipStream_t s)
{
    hipLaunchKernelGGL(zero_word_kernel, dim3(1), dim3(1), 0, s, flag);
    const unsigned blocks = (unsigned)std::min<size_t>(1024, ceil_div((int64_t)std::max<size_t>(count, 1), 256));
    hipLaunchKernelGGL(check_inputs_kernel, dim3(blocks), dim3(256), 0, s, lo, hi, count, label, batch, nK, flag);
    DPC_HIP(hipGetLastError());
    int32_t h = 0;
    DPC_HIP(hipMemcpyAsync(&h, flag, sizeof h, hipMemcpyDeviceToHost, s));
    DPC_HIP(hipStreamSynchronize(s));
    return (h & 1) ? 1 : (h & 2) ? 2 : 0;
}

void ingest_enqueue(const float* lo, const float* hi, const int32_t* label, float* l0, float* u0, int32_t* lab, int batch, int n0,
                    int Cc, int H, int W, int nK, int32_t* flag, int32_t* pinned_host_flag, hipStream_t s, float* pk, int ld)
{
    if (!pk) ld = n0;
    DPC_REQUIRE(ld >= n0 && ((uintptr_t)pk % 16) == 0, DPC_EINVAL, "ingest: bad arguments");
    const size_t count = (size_t)batch * ld;
    const unsigned blocks = (unsigned)std::min<size_t>(1024, ceil_div((int64_t)std::max<size_t>(count, 1), 256));
    hipLaunchKernelGGL(ingest_kernel, dim3(blocks), dim3(256), 0, s, lo, hi, label, l0, u0, lab, batch, n0, Cc, H, W, nK, flag,
                       reinterpret_cast<float4*>(pk), ld);
    DPC_HIP(hipGetLastError());
    DPC_HIP(hipMemcpyAsync(pinned_host_flag, flag, sizeof(int32_t), hipMemcpyDeviceToHost, s));
}

void zero_word_enqueue(int32_t* flag, hipStream_t s)
{
    hipLaunchKernelGGL(zero_word_kernel, dim3(1), dim3(1), 0, s, flag);
    DPC_HIP(hipGetLastError());
}

void check_inputs_enqueue(const float* lo, const float* hi, size_t count, const int32_t* label, int batch, int nK,
                          int32_t* flag, int32_t* pinned_host_flag, hipStream_t s)
{
    hipLaunchKernelGGL(zero_word_kernel, dim3(1), dim3(1), 0, s, flag);
    const unsigned blocks = (unsigned)std::min<size_t>(1024, ceil_div((int64_t)std::max<size_t>(count, 1), 256));
    hipLaunchKernelGGL(check_inputs_kernel, dim3(blocks), dim3(256), 0, s, lo, hi, count, label, batch, nK, flag);
    DPC_HIP(hipGetLastError());
    DPC_HIP(hipMemcpyAsync(pinned_host_flag, flag, sizeof(int32_t), hipMemcpyDeviceToHost, s));
}

}  // namespace dpc
