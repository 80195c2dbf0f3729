// ReuseCert (Appendix C, "ReuseCert"; Section 6.1): every affine layer keeps its polyhedral bounds already
// back-substituted to the input layer, so a later layer's traversal is ONE replacement step
//     lower_k = W+ * Lr + W- * Ur + b,   upper_k = W+ * Ur + W- * Lr + b,
// where Lr, Ur are the ReLU layer's bounds over the input: Lr_j = lambda_j * L_j, Ur_j = mu_j * U_j + nu_j.
//
// Layout: an input-level expression is a row of ldE = round_up(n0 + 1, 32) floats, coefficients over the n0
// inputs followed by the constant in column n0.  Stored bounds of layer k: E[side][b][r] (side 0 = L, 1 = U).
// The replacement step is a contraction  [W+ | W- | b] (shared, [n_k, 2 n_{k-1} + 1])  x  Rr[b]
// ([2 n_{k-1} + 1, ldE] per input: rows Lr, then Ur, then the unit row that carries the bias), batched over
// the inputs; the helpers here build those two operands.
#include "common.h"
#include "conv.h"

namespace dpc {

namespace {

constexpr int kThreads = 256;
typedef float vf4 __attribute__((ext_vector_type(4)));

// Rr[b][j]       = lambda[b][j] * L_j            (j < n)
// Rr[b][n + j]   = mu[b][j] * U_j + nu[b][j] e_n0
// Rr[b][2n]      = e_n0
// SHARED: L_j = U_j = (W1[j], bias[j]) for every input (first layer); otherwise rows of E.
template <bool SHARED>
__global__ __launch_bounds__(kThreads) void reuse_scale_kernel(
    const float* __restrict__ E, const float* __restrict__ W1, int ldw, const float* __restrict__ bias,
    const float* __restrict__ lambda, const float* __restrict__ mu, const float* __restrict__ nu,
    int batch, int n, int n0, int ldE, float* __restrict__ Rr, int mod)
{
    const int b = blockIdx.y;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int j = blockIdx.x * (kThreads / 64) + wave;
    if (j > 2 * n) return;
    float* dst = Rr + ((size_t)b * (2 * n + 1) + j) * ldE;
    if (j == 2 * n) {
        for (int c = lane * 4; c < ldE; c += 256) {
            vf4 o = {0.f, 0.f, 0.f, 0.f};
            if (n0 >= c && n0 < c + 4) o[n0 - c] = 1.0f;
            *reinterpret_cast<vf4*>(dst + c) = o;
        }
        return;
    }
    const int side = j >= n, jj = side ? j - n : j;
    const float scale = side ? mu[(size_t)b * n + jj] : lambda[(size_t)b * n + jj];
    const float add = side ? nu[(size_t)b * n + jj] : 0.0f;
    const float* src = SHARED ? W1 + (size_t)(jj % mod) * ldw : E + (((size_t)side * batch + b) * n + jj) * ldE;
    const float cst = SHARED ? bias[jj % mod] : 0.0f;
    for (int c = lane * 4; c < ldE; c += 256) {
        vf4 x = {0.f, 0.f, 0.f, 0.f};
        if (SHARED) {
#pragma unroll
            for (int t = 0; t < 4; ++t) x[t] = c + t < n0 ? src[c + t] : (c + t == n0 ? cst : 0.0f);
        } else {
            x = *reinterpret_cast<const vf4*>(src + c);
        }
        vf4 o;
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = scale * x[t] + (c + t == n0 ? add : 0.0f);
        *reinterpret_cast<vf4*>(dst + c) = o;
    }
}

// dst[m] = [ c+ | c- | constant ] (lower side) or [ c- | c+ | constant ] (upper side) of row m of src, c+ = max(c, 0),
// c- = min(c, 0); columns 2n+1 .. ld_dst-1 zero.  side = m / rows_per_side when rows_per_side > 0, else `side0`.
__global__ __launch_bounds__(kThreads) void reuse_split_kernel(
    const float* __restrict__ src, int ld_src, const float* __restrict__ bias_f, const double* __restrict__ bias_d,
    long long rows, int n, float* __restrict__ dst, int ld_dst, long long rows_per_side, int side0)
{
    const long long m = (long long)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (m >= rows) return;
    const int side = rows_per_side > 0 ? (int)(m / rows_per_side) : side0;
    const float* in = src + m * ld_src;
    float* out = dst + m * ld_dst;
    const float cst = bias_d ? (float)bias_d[m] : bias_f[m];
    for (int c = lane; c < ld_dst; c += 64) {
        float v = 0.0f;
        if (c < 2 * n) {
            const float w = in[c < n ? c : c - n];
            const bool first = c < n;                           // first half multiplies Lr, second half Ur
            const bool take_pos = (side == 0) == first;         // lower: c+ on Lr, c- on Ur; upper: mirrored
            v = take_pos ? fmaxf(w, 0.0f) : fminf(w, 0.0f);
        } else if (c == 2 * n) {
            v = cst;
        }
        out[c] = v;
    }
}

__global__ __launch_bounds__(kThreads) void reuse_const_kernel(const float* __restrict__ C, int ldc, int col, long long rows,
                                                              double* __restrict__ cst)
{
    const long long m = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (m < rows) cst[m] = (double)C[m * ldc + col];
}

// Right operand of the replacement step through a convolution layer (the layer's weight matrix is its expanded kernel:
// neuron (ho, wo, co) reads the kh x kw x Ci window at (ho*S - P, wo*S - P) of the ReLU layer below).  For output
// position z = (b, ho, wo) the rows of Rr[b] that window touches are gathered in the order of the split kernel matrix
// [K+ | K- | b] = (ky, kx, ci) over Lr, the same over Ur, then the unit row:
//   G[z - z0][k] = Lr / Ur row of neuron ((y*W + x)*Ci + ci), zeros where the window hangs over the zero padding.
// One workgroup per (position, row).
__global__ __launch_bounds__(kThreads) void reuse_gather_kernel(const float* __restrict__ Rr, int n, int ldE, ConvGeom g,
                                                               long long z0, float* __restrict__ G, int Kp)
{
    const long long z = z0 + blockIdx.x;
    const int k = blockIdx.y;
    const int npos = g.Ho * g.Wo, kk = g.kh * g.kw * g.Ci;
    const int b = (int)(z / npos), pos = (int)(z - (long long)b * npos);
    const int ho = pos / g.Wo, wo = pos - ho * g.Wo;
    const float* src = nullptr;
    const float* base = Rr + (size_t)b * (2 * (size_t)n + 1) * ldE;
    if (k == 2 * kk) {
        src = base + (size_t)2 * n * ldE;
    } else {
        const int part = k >= kk, kt = part ? k - kk : k;
        const int ci = kt % g.Ci, kx = (kt / g.Ci) % g.kw, ky = kt / (g.Ci * g.kw);
        const int y = ho * g.stride - g.pad + ky, x = wo * g.stride - g.pad + kx;
        if (y >= 0 && y < g.H && x >= 0 && x < g.W) src = base + ((size_t)part * n + ((size_t)y * g.W + x) * g.Ci + ci) * ldE;
    }
    float* dst = G + ((size_t)blockIdx.x * Kp + k) * ldE;
    for (int c = threadIdx.x * 4; c < ldE; c += kThreads * 4) {
        vf4 v = {0.f, 0.f, 0.f, 0.f};
        if (src) v = *reinterpret_cast<const vf4*>(src + c);
        *reinterpret_cast<vf4*>(dst + c) = v;
    }
}

// ---- stored bounds of convolution layers in patch form -------------------------------------------------------
// The stored input-level bounds of a convolution neuron (y, x, c) only reach its receptive field: a window of
// ph x pw x C0 input positions whose corner is (y*S - P, x*S - P) (C0 = channels of the network input; positions off the
// image carry no input and are ignored by every consumer).  A row holds the window's coefficients followed by the
// constant in column ph*pw*C0.  All neurons of one position share a window, so the replacement step through the next
// convolution layer is again one contraction per output position, with the rows it gathers embedded in the (larger)
// window of that position: tap (ky, kx) of the layer sits at offset (ky*S, kx*S) of it.
struct RWin { int ph, pw, C0, S, P, ld; };      // ld: floats per row (>= ph*pw*C0 + 1)

__global__ __launch_bounds__(kThreads) void reuse_gather_patch_kernel(const float* __restrict__ Rr, int n, RWin fi, RWin fo, ConvGeom g,
                                                                     long long z0, float* __restrict__ G, int Kp)
{
    const long long z = z0 + blockIdx.x;
    const int k = blockIdx.y;
    const int npos = g.Ho * g.Wo, kk = g.kh * g.kw * g.Ci;
    const int b = (int)(z / npos), pos = (int)(z - (long long)b * npos);
    const int ho = pos / g.Wo, wo = pos - ho * g.Wo;
    const float* base = Rr + (size_t)b * (2 * (size_t)n + 1) * fi.ld;
    const int ei = fi.ph * fi.pw * fi.C0, eo = fo.ph * fo.pw * fo.C0;
    float* dst = G + ((size_t)blockIdx.x * Kp + k) * fo.ld;
    if (k == 2 * kk) {                                               // unit row: carries the bias
        for (int e = threadIdx.x; e < fo.ld; e += kThreads) dst[e] = e == eo ? 1.0f : 0.0f;
        return;
    }
    const int part = k >= kk, kt = part ? k - kk : k;
    const int ci = kt % g.Ci, kx = (kt / g.Ci) % g.kw, ky = kt / (g.Ci * g.kw);
    const int y = ho * g.stride - g.pad + ky, x = wo * g.stride - g.pad + kx;
    const bool on = y >= 0 && y < g.H && x >= 0 && x < g.W;          // off the layer's grid: zero padding, no neuron
    const float* src = base + ((size_t)part * n + ((size_t)y * g.W + x) * g.Ci + ci) * fi.ld;
    const int dy = ky * fi.S, dx = kx * fi.S;
    for (int e = threadIdx.x; e < fo.ld; e += kThreads) {
        float v = 0.0f;
        if (on) {
            if (e < eo) {
                const int c = e % fo.C0, q = e / fo.C0;
                const int qx = q % fo.pw, qy = q / fo.pw;
                const int py = qy - dy, px = qx - dx;
                if (py >= 0 && py < fi.ph && px >= 0 && px < fi.pw) v = src[(py * fi.pw + px) * fi.C0 + c];
            } else if (e == eo) {
                v = src[ei];
            }
        }
        dst[e] = v;
    }
}

// Rr[b][j] (dense rows over the input, constant in column n0) from stored bounds in patch form: row j < n is
// lambda * L_j, row n + j is mu * U_j + nu, row 2n the unit row, written out over the whole input for the
// fully-connected layer that follows the last convolution.  SHARED: L_j = U_j = (core[j % mod], bias[j % mod]).
template <bool SHARED>
__global__ __launch_bounds__(kThreads) void reuse_scale_expand_kernel(
    const float* __restrict__ E, const float* __restrict__ core, int ld_core, const float* __restrict__ bias, int mod,
    const float* __restrict__ lambda, const float* __restrict__ mu, const float* __restrict__ nu, int batch, int n, RWin fi,
    int rows_W, int rows_C, int gh, int gw, int n0, int ldE, float* __restrict__ Rr)
{
    const int b = blockIdx.y, j = blockIdx.x;
    float* dst = Rr + ((size_t)b * (2 * n + 1) + j) * ldE;
    if (j == 2 * n) {
        for (int e = threadIdx.x; e < ldE; e += kThreads) dst[e] = e == n0 ? 1.0f : 0.0f;
        return;
    }
    const int side = j >= n, jj = side ? j - n : j;
    const float scale = side ? mu[(size_t)b * n + jj] : lambda[(size_t)b * n + jj];
    const float add = side ? nu[(size_t)b * n + jj] : 0.0f;
    const float* src = SHARED ? core + (size_t)(jj % mod) * ld_core : E + (((size_t)side * batch + b) * n + jj) * fi.ld;
    const float cst = SHARED ? bias[jj % mod] : src[fi.ph * fi.pw * fi.C0];
    const int wo = (jj / rows_C) % rows_W, ho = jj / (rows_C * rows_W);
    const int oy = ho * fi.S - fi.P, ox = wo * fi.S - fi.P;
    for (int e = threadIdx.x; e < ldE; e += kThreads) {
        float v = 0.0f;
        if (e < n0) {
            const int c = e % fi.C0, q = e / fi.C0;
            const int gx = q % gw, gy = q / gw;
            const int py = gy - oy, px = gx - ox;
            if (py >= 0 && py < fi.ph && px >= 0 && px < fi.pw) v = scale * src[(py * fi.pw + px) * fi.C0 + c];
        } else if (e == n0) {
            v = scale * cst + add;
        }
        dst[e] = v;
    }
}

}  // namespace

void launch_reuse_scale(const float* E, const float* W1, int ldw, const float* bias, const float* lambda, const float* mu,
                        const float* nu, int batch, int n, int n0, int ldE, float* Rr, hipStream_t s, int mod)
{
    if (mod <= 0) mod = n;
    DPC_REQUIRE(lambda && mu && nu && Rr && (E || (W1 && bias)) && n >= 1 && n0 >= 1 && ldE > n0 && ldE % 4 == 0 &&
                    batch >= 0 && batch <= 65535, DPC_EINVAL, "reuse_scale: bad arguments");
    DPC_REQUIRE(E || ldw >= n0, DPC_EINVAL, "reuse_scale: weight rows too short");
    DPC_REQUIRE(((uintptr_t)Rr % 16) == 0 && (!E || ((uintptr_t)E % 16) == 0), DPC_EINVAL, "reuse_scale: buffers must be 16-byte aligned");
    if (batch == 0) return;
    dim3 grid((unsigned)ceil_div(2 * n + 1, kThreads / 64), (unsigned)batch);
    if (E)
        hipLaunchKernelGGL(reuse_scale_kernel<false>, grid, dim3(kThreads), 0, s, E, (const float*)nullptr, 0, (const float*)nullptr,
                           lambda, mu, nu, batch, n, n0, ldE, Rr, mod);
    else
        hipLaunchKernelGGL(reuse_scale_kernel<true>, grid, dim3(kThreads), 0, s, (const float*)nullptr, W1, ldw, bias, lambda, mu,
                           nu, batch, n, n0, ldE, Rr, mod);
    DPC_HIP(hipGetLastError());
}

void launch_reuse_split(const float* src, int ld_src, const float* bias_f, const double* bias_d, int64_t rows, int n,
                        float* dst, int ld_dst, int64_t rows_per_side, int side0, hipStream_t s)
{
    DPC_REQUIRE(src && dst && (bias_f || bias_d) && rows >= 0 && n >= 1 && ld_src >= n && ld_dst >= 2 * n + 1, DPC_EINVAL,
                "reuse_split: bad arguments");
    if (rows == 0) return;
    hipLaunchKernelGGL(reuse_split_kernel, dim3((unsigned)ceil_div(rows, kThreads / 64)), dim3(kThreads), 0, s, src, ld_src, bias_f,
                       bias_d, (long long)rows, n, dst, ld_dst, (long long)rows_per_side, side0);
    DPC_HIP(hipGetLastError());
}

void launch_reuse_const(const float* C, int ldc, int col, int64_t rows, double* cst, hipStream_t s)
{
    DPC_REQUIRE(C && cst && col >= 0 && col < ldc && rows >= 0, DPC_EINVAL, "reuse_const: bad arguments");
    if (rows == 0) return;
    hipLaunchKernelGGL(reuse_const_kernel, dim3((unsigned)ceil_div(rows, kThreads)), dim3(kThreads), 0, s, C, ldc, col,
                       (long long)rows, cst);
    DPC_HIP(hipGetLastError());
}

void launch_reuse_gather(const float* Rr, int n, int ldE, const ConvGeom& g, int64_t z0, int64_t nz, float* G, hipStream_t s)
{
    const int Kp = 2 * g.kh * g.kw * g.Ci + 1;
    DPC_REQUIRE(Rr && G && n == g.Ci * g.H * g.W && ldE % 4 == 0 && z0 >= 0 && nz >= 0 && nz <= 0x7fffffff && Kp <= 65535, DPC_EINVAL,
                "reuse_gather: bad arguments");
    DPC_REQUIRE(((uintptr_t)Rr % 16) == 0 && ((uintptr_t)G % 16) == 0, DPC_EINVAL, "reuse_gather: buffers must be 16-byte aligned");
    if (nz == 0) return;
    hipLaunchKernelGGL(reuse_gather_kernel, dim3((unsigned)nz, (unsigned)Kp), dim3(kThreads), 0, s, Rr, n, ldE, g, (long long)z0, G, Kp);
    DPC_HIP(hipGetLastError());
}

void launch_reuse_gather_patch(const float* Rr, int n, const ReuseWindow& fi, const ReuseWindow& fo, const ConvGeom& g, int64_t z0,
                               int64_t nz, float* G, hipStream_t s)
{
    const int Kp = 2 * g.kh * g.kw * g.Ci + 1;
    DPC_REQUIRE(Rr && G && n == g.Ci * g.H * g.W && z0 >= 0 && nz >= 0 && nz <= 0x7fffffff && Kp <= 65535, DPC_EINVAL,
                "reuse_gather_patch: bad arguments");
    DPC_REQUIRE(fi.C0 == fo.C0 && fo.ph == (g.kh - 1) * fi.S + fi.ph && fo.pw == (g.kw - 1) * fi.S + fi.pw &&
                    fi.ld > fi.ph * fi.pw * fi.C0 && fo.ld > fo.ph * fo.pw * fo.C0, DPC_EINVAL, "reuse_gather_patch: windows do not fit");
    if (nz == 0) return;
    const RWin a{fi.ph, fi.pw, fi.C0, fi.S, fi.P, fi.ld}, o{fo.ph, fo.pw, fo.C0, fo.S, fo.P, fo.ld};
    hipLaunchKernelGGL(reuse_gather_patch_kernel, dim3((unsigned)nz, (unsigned)Kp), dim3(kThreads), 0, s, Rr, n, a, o, g, (long long)z0, G, Kp);
    DPC_HIP(hipGetLastError());
}

void launch_reuse_scale_expand(const float* E, const float* core, int ld_core, const float* bias, int mod, const float* lambda,
                               const float* mu, const float* nu, int batch, int n, const ReuseWindow& fi, int rows_W, int rows_C, int gh,
                               int gw, int n0, int ldE, float* Rr, hipStream_t s)
{
    DPC_REQUIRE(lambda && mu && nu && Rr && (E || (core && bias && mod >= 1)) && n >= 1 && n0 == gh * gw * fi.C0 && ldE > n0 && batch >= 0 &&
                    batch <= 65535 && n == (n / (rows_W * rows_C)) * rows_W * rows_C, DPC_EINVAL, "reuse_scale_expand: bad arguments");
    if (batch == 0) return;
    const RWin a{fi.ph, fi.pw, fi.C0, fi.S, fi.P, fi.ld};
    dim3 grid((unsigned)(2 * n + 1), (unsigned)batch);
    if (E)
        hipLaunchKernelGGL(reuse_scale_expand_kernel<false>, grid, dim3(kThreads), 0, s, E, (const float*)nullptr, 0, (const float*)nullptr, 1,
                           lambda, mu, nu, batch, n, a, rows_W, rows_C, gh, gw, n0, ldE, Rr);
    else
        hipLaunchKernelGGL(reuse_scale_expand_kernel<true>, grid, dim3(kThreads), 0, s, (const float*)nullptr, core, ld_core, bias, mod, lambda,
                           mu, nu, batch, n, a, rows_W, rows_C, gh, gw, n0, ldE, Rr);
    DPC_HIP(hipGetLastError());
}

}  // namespace dpc
