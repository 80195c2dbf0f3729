// Split-precision contraction (throughput experiment, off by default): Cout = A * W with both operands written as
// sums of TERMS bf16 numbers (x = x0 + x1 [+ x2], each the bf16 rounding of what the previous ones left) and the
// product formed on the bf16 MFMA units from the partial products whose orders add up to less than TERMS:
//   TERMS = 2: x0*w0 + x0*w1 + x1*w0            ("bf16x3", about 16 significand bits per product)
//   TERMS = 3: the six products of order <= 2    ("bf16x6", about 24 bits: fp32-like)
// accumulated in fp32.  v_mfma_f32_32x32x16_bf16 runs 16 times the multiply-adds per cycle of the fp32 MFMA, so three
// (six) of them per tile still leave 5.3x (2.7x) the fp32 peak.  The weights are split once per network into
// Wt[term][n][k] (transposed: a B-operand lane wants 8 consecutive k of one column); the rows are split when a tile
// is staged in LDS.
//
// Workgroup: 256 threads = 2 x 2 wavefronts, tile 128 x 128 or 128 x 256, K step 32; a wavefront owns 64 x 64 or
// 64 x 128 (2 x 2 or 2 x 4 MFMA tiles; the wide tile converts the rows once for twice the columns).
// Operand lanes of the 32x32x16 MFMA: lane l holds row (column) l % 32 and k = 8 * (l / 32) .. + 7.
#include <algorithm>

#include "common.h"

namespace dpc {

int contract_split_terms() { return tune(TK_CONTRACT_SPLIT); }

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float vf2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float vf4 __attribute__((ext_vector_type(4)));
typedef unsigned vu4 __attribute__((ext_vector_type(4)));

constexpr int kBM = 128, kBK = 32, kNPad = 256;
// LDS tiles are [k chunk of 8 bf16 = 16 B][row]: the 32 lanes of a half-wave read consecutive 16-byte units; planes are
// rows + 4 units apart (16 banks mod 64), which also keeps the staging writes below free of bank conflicts

template <int TERMS>
__device__ __forceinline__ void split(float x, __bf16 (&o)[TERMS])
{
    float r = x;
#pragma unroll
    for (int t = 0; t < TERMS; ++t) {
        o[t] = (__bf16)r;
        r -= (float)o[t];
    }
}

// Wt[t][n][k] = term t of W[k][n]; rows n >= N and columns k >= K of Wt are zero (set by the caller).
template <int TERMS>
__global__ __launch_bounds__(256) void split_weights_kernel(const float* __restrict__ W, int K, int N, int ldw,
                                                            __bf16* __restrict__ Wt, int ldk, size_t term_stride)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;       // over [K][N], n fastest (coalesced reads)
    if (i >= (int64_t)K * N) return;
    const int n = (int)(i % N), k = (int)(i / N);
    __bf16 p[TERMS];
    split<TERMS>(W[(size_t)k * ldw + n], p);
#pragma unroll
    for (int t = 0; t < TERMS; ++t) Wt[t * term_stride + (size_t)n * ldk + k] = p[t];
}

// Epilogue arguments of the fused variant (EPI = 1): the traversal step that follows the contraction -- sign-split ReLU
// step of the layer below or the concretisation at the input -- applied to the accumulators from packed parameters
// pk[g][c] = (pm, nm, kp, kn), g = row / R: stored value x * (x >= 0 ? pm : nm), row constant += x * (x >= 0 ? kp : kn).
// Row-constant partial sums: fixed-order reduction over the tile's columns, one slot per column tile.
struct SplitEpi {
    const float4* pk;
    int ldpk, R, nsb;
    float* part;
    long long part_stride;
    int store;
};

template <int NTW>
__device__ __forceinline__ void store_cols(float* dst, const float (&o)[NTW])
{
    if constexpr (NTW == 2) *reinterpret_cast<float2*>(dst) = make_float2(o[0], o[1]);
    else *reinterpret_cast<float4*>(dst) = make_float4(o[0], o[1], o[2], o[3]);
}

// NTW: MFMA tiles of 32 columns per wavefront (2 or 4); the workgroup tile is 128 x (64 * NTW).
template <int TERMS, int EPI, int NTW>
__global__ __launch_bounds__(256, (TERMS == 2 && NTW == 2) ? 3 : 2) void contract_split_kernel(
    const float* __restrict__ A, long long M, int K, int lda, const __bf16* __restrict__ Wt, int ldk, size_t term_stride,
    int N, float* __restrict__ C, int ldc, int tiles_m, int tiles_n, SplitEpi ep)
{
    constexpr int BN = 64 * NTW, WN = 32 * NTW, BQ = BN / 64;
    __shared__ __attribute__((aligned(16))) vu4 sA[TERMS][4][kBM + 4];
    __shared__ __attribute__((aligned(16))) vu4 sB[TERMS][4][BN + 4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, kq = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    // XCD-aware order (workgroup ids go round-robin over the 8 XCDs; gridDim.x is a multiple of 8): the column tiles
    // of one row tile run on one XCD, so its L2 serves the re-reads of the rows
    const int per_xcd = gridDim.x >> 3;
    const int v = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (v >= tiles_m * tiles_n) return;
    const int tm = v / tiles_n, tn = v - tm * tiles_n;
    const long long m0 = (long long)tm * kBM;
    const int n0 = tn * BN;
    // Staging.  Rows: thread t brings 4 consecutive k (piece t % 8 of the 32) of rows t / 8 + 32 q, q < 4: 8 lanes read
    // one 128-byte run.  Weights: thread t brings chunk t % 4 (8 k, 16 B) of the columns held by LDS rows t / 4 + 64 q.
    // A wavefront's MFMA tile j holds the columns NTW * l + j of its WN (a lane then owns NTW adjacent columns and stores
    // them as one vector), i.e. LDS row b of a wavefront's block holds column NTW * (b % 32) + b / 32 of that block.
    const int arow = tid >> 3, apiece = tid & 7;
    const int bb = tid >> 2, bchunk = tid & 3;
    // Both operands come through buffer loads: the K offset is a scalar, a lane's byte offset is fixed for the whole
    // loop, and an offset outside the resource returns zeros -- rows past M need neither a branch nor a zero fill.
    // The resources start at this workgroup's first row / column so that 32-bit offsets suffice.
    const long long arows = M - m0 < kBM ? M - m0 : kBM;
    const __amdgpu_buffer_rsrc_t ares = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(A + m0 * (long long)lda), 0, (int)(((arows - 1) * lda + K) * 4), 0x00020000);
    const __amdgpu_buffer_rsrc_t bres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<__bf16*>(Wt + (size_t)n0 * ldk), 0, (int)(((size_t)(TERMS - 1) * term_stride + (size_t)BN * ldk) * 2), 0x00020000);
    constexpr int kOutside = (int)0x80000000;
    int aoff[4], boff[TERMS][BQ];
#pragma unroll
    for (int q = 0; q < 4; ++q) aoff[q] = arow + 32 * q < arows ? ((arow + 32 * q) * lda + 4 * apiece) * 4 : kOutside;
#pragma unroll
    for (int q = 0; q < BQ; ++q) {
        const int r = bb + 64 * q, blk = r / WN, b = r - blk * WN;
        const int col = blk * WN + NTW * (b & 31) + (b >> 5);
#pragma unroll
        for (int t = 0; t < TERMS; ++t) boff[t][q] = (int)((t * term_stride + (size_t)col * ldk + 8 * bchunk) * 2);
    }

    floatx16 acc[2][NTW];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < NTW; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    vf4 ra[4];
    vu4 rb[TERMS][BQ];
    auto fetch = [&](int kt) __attribute__((always_inline)) {
        const int k0 = kt * kBK;
        const bool kin = k0 + 4 * apiece < K;                  // K is a multiple of 4; only the last step can leave the rows
#pragma unroll
        for (int q = 0; q < 4; ++q)
            ra[q] = __builtin_bit_cast(vf4, __builtin_amdgcn_raw_buffer_load_b128(ares, kin ? aoff[q] : kOutside, k0 * 4, 0));
#pragma unroll
        for (int t = 0; t < TERMS; ++t)
#pragma unroll
            for (int q = 0; q < BQ; ++q) rb[t][q] = __builtin_amdgcn_raw_buffer_load_b128(bres, boff[t][q], k0 * 2, 0);   // ldk covers the padded K
    };
    const int nk = (K + kBK - 1) / kBK;
    fetch(0);
    for (int kt = 0; kt < nk; ++kt) {
        // registers -> LDS (rows split into their bf16 terms on the way)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            vf2 r01 = {ra[q][0], ra[q][1]}, r23 = {ra[q][2], ra[q][3]};
#pragma unroll
            for (int t = 0; t < TERMS; ++t) {
                // two elements per conversion instruction; a bf16 widened back to fp32 is its bits shifted up
                const bf16x2 p01 = __builtin_convertvector(r01, bf16x2), p23 = __builtin_convertvector(r23, bf16x2);
                const unsigned b01 = __builtin_bit_cast(unsigned, p01), b23 = __builtin_bit_cast(unsigned, p23);
                if (t + 1 < TERMS) {
                    r01[0] -= __uint_as_float(b01 << 16); r01[1] -= __uint_as_float(b01 & 0xffff0000u);
                    r23[0] -= __uint_as_float(b23 << 16); r23[1] -= __uint_as_float(b23 & 0xffff0000u);
                }
                // piece = half a 16-byte chunk
                uint2* dst = reinterpret_cast<uint2*>(&sA[t][apiece >> 1][arow + 32 * q]) + (apiece & 1);
                *dst = make_uint2(b01, b23);
            }
        }
#pragma unroll
        for (int t = 0; t < TERMS; ++t)
#pragma unroll
            for (int q = 0; q < BQ; ++q) sB[t][bchunk][bb + 64 * q] = rb[t][q];
        __syncthreads();
        if (kt + 1 < nk) fetch(kt + 1);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 a[TERMS][2], b[TERMS][NTW];
#pragma unroll
            for (int t = 0; t < TERMS; ++t) {
#pragma unroll
                for (int i = 0; i < 2; ++i) a[t][i] = __builtin_bit_cast(bf16x8, sA[t][2 * ks + kq][wm * 64 + i * 32 + l32]);
#pragma unroll
                for (int j = 0; j < NTW; ++j) b[t][j] = __builtin_bit_cast(bf16x8, sB[t][2 * ks + kq][wn * WN + j * 32 + l32]);
            }
            // smallest partial products first
#pragma unroll
            for (int order = TERMS - 1; order >= 0; --order)
#pragma unroll
                for (int ta = 0; ta <= order; ++ta)
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int j = 0; j < NTW; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ta][i], b[order - ta][j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // accumulator register 4*i4 + j4 of a lane is row 8*i4 + 4*(lane/32) + j4 of its MFMA tile; the lane's columns
    // are NTW*l32 .. NTW*l32 + NTW-1 of the wavefront's block (tiles j = 0 .. NTW-1)
    const int col = n0 + wn * WN + NTW * l32;
    if constexpr (EPI == 0) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const long long row = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * kq + (r & 3);
                if (row < M && col < ldc) {            // ldc is a multiple of 4; padding columns are kept at zero
                    float o[NTW];
#pragma unroll
                    for (int j = 0; j < NTW; ++j) o[j] = col + j < N ? acc[i][j][r] : 0.0f;
                    store_cols<NTW>(C + row * ldc + col, o);
                }
            }
    } else {
        float* sRow = reinterpret_cast<float*>(&sA[0][0][0]);          // [2][kBM]: the K loop is done with LDS
        const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const long long rb0 = m0 + wm * 64 + i * 32;
            const long long rclamp = rb0 < M ? rb0 : M - 1;
            const int g_lo = (int)(rclamp / ep.R);
            const long long boundary = (long long)(g_lo + 1) * ep.R;     // first row of the next group
            const bool two = boundary < rb0 + 32;                        // wave-uniform; R >= 32: at most one boundary
            const int g_hi = g_lo + 1 < ep.nsb ? g_lo + 1 : ep.nsb - 1;
            float4 pa[NTW], pb[NTW];
#pragma unroll
            for (int j = 0; j < NTW; ++j) {
                const bool ok = col + j < ep.ldpk;
                pa[j] = ok ? ep.pk[(size_t)g_lo * ep.ldpk + col + j] : zero4;
                pb[j] = (ok && two) ? ep.pk[(size_t)g_hi * ep.ldpk + col + j] : pa[j];
            }
            float rs[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const long long row = rb0 + 8 * (r >> 2) + 4 * kq + (r & 3);
                const bool useb = row >= boundary;
                float o[NTW];
                float sum = 0.0f;
#pragma unroll
                for (int j = 0; j < NTW; ++j) {
                    const float x = acc[i][j][r];
                    const float4 Pm = useb ? pb[j] : pa[j];
                    const bool pos = x >= 0.0f;
                    o[j] = x * (pos ? Pm.x : Pm.y);
                    sum += x * (pos ? Pm.z : Pm.w);
                }
                rs[r] = sum;
                if (ep.store && row < M && col < ldc) store_cols<NTW>(C + row * ldc + col, o);
            }
            // butterfly with halving over the 32 lanes that share these rows (fixed order): after the steps with
            // lane bits 0..3 a lane holds the sum over its 16-lane group of one register index, the last step adds
            // the two groups
            float v8[8], v4[4], v2[2], v1;
            {
                const bool h = l32 & 1;
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const float send = h ? rs[k] : rs[k + 8];
                    const float keep = h ? rs[k + 8] : rs[k];
                    v8[k] = keep + __shfl_xor(send, 1, 64);
                }
            }
            {
                const bool h = l32 & 2;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float send = h ? v8[k] : v8[k + 4];
                    const float keep = h ? v8[k + 4] : v8[k];
                    v4[k] = keep + __shfl_xor(send, 2, 64);
                }
            }
            {
                const bool h = l32 & 4;
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    const float send = h ? v4[k] : v4[k + 2];
                    const float keep = h ? v4[k + 2] : v4[k];
                    v2[k] = keep + __shfl_xor(send, 4, 64);
                }
            }
            {
                const bool h = l32 & 8;
                const float send = h ? v2[0] : v2[1];
                const float keep = h ? v2[1] : v2[0];
                v1 = keep + __shfl_xor(send, 8, 64);
            }
            v1 += __shfl_xor(v1, 16, 64);
            if (l32 < 16) {
                const int vv = 8 * (l32 & 1) + 4 * ((l32 >> 1) & 1) + 2 * ((l32 >> 2) & 1) + ((l32 >> 3) & 1);
                sRow[wn * kBM + wm * 64 + i * 32 + 8 * (vv >> 2) + 4 * kq + (vv & 3)] = v1;
            }
        }
        __syncthreads();
        for (int r = tid; r < kBM; r += 256) {
            const float t = sRow[r] + sRow[kBM + r];
            if (m0 + r < M) ep.part[(size_t)tn * ep.part_stride + m0 + r] = t;
        }
    }
}

}  // namespace

size_t split_weights_elems(int K, int N, int terms, int* ldk, int* npad)
{
    *ldk = (int)round_up(K, kBK);
    *npad = (int)round_up(N, kNPad);
    return (size_t)terms * *npad * *ldk;
}

void launch_split_weights(const float* W, int K, int N, int ldw, int terms, void* Wt, hipStream_t s)
{
    DPC_REQUIRE(W && Wt && (terms == 2 || terms == 3) && K >= 1 && N >= 1 && ldw >= N, DPC_EINVAL, "split_weights: bad arguments");
    int ldk, npad;
    const size_t elems = split_weights_elems(K, N, terms, &ldk, &npad);
    DPC_HIP(hipMemsetAsync(Wt, 0, elems * 2, s));
    const size_t ts = (size_t)npad * ldk;
    const unsigned grid = (unsigned)ceil_div((int64_t)K * N, 256);
    if (terms == 2)
        hipLaunchKernelGGL(split_weights_kernel<2>, dim3(grid), dim3(256), 0, s, W, K, N, ldw, reinterpret_cast<__bf16*>(Wt), ldk, ts);
    else
        hipLaunchKernelGGL(split_weights_kernel<3>, dim3(grid), dim3(256), 0, s, W, K, N, ldw, reinterpret_cast<__bf16*>(Wt), ldk, ts);
    DPC_HIP(hipGetLastError());
}

namespace {

// 256-column tiles unless the last one would be at most half used (e.g. 784 columns)
int pick_ntw(int ldc)
{
    if (tune(TK_CONTRACT_SPLIT_WIDE) >= 0) return tune(TK_CONTRACT_SPLIT_WIDE) ? 4 : 2;     // -1: 256-column tiles by shape
    const int rem = ldc % 256;
    return (rem != 0 && rem <= 128) ? 2 : 4;
}

template <int EPI>
int launch_split_kernel(const float* A, int64_t M, int K, int lda, const void* Wt, int terms, int N, float* C, int ldc,
                        const SplitEpi& ep, int max_slots, hipStream_t s)
{
    int ldk, npad;
    split_weights_elems(K, N, terms, &ldk, &npad);
    const int ntw = terms == 2 ? pick_ntw(ldc) : 2;     // three terms with the wide tile would not fit registers and LDS
    const int64_t tiles_m = ceil_div(M, kBM);
    const int tiles_n = (int)ceil_div(ldc, 64 * ntw);                      // padding columns of C are written too
    DPC_REQUIRE(tiles_m * tiles_n < ((int64_t)1 << 30), DPC_EINVAL, "contract_split: too many tiles");
    if (EPI == 1 && tiles_n > max_slots) return -1;
    const dim3 grid((unsigned)round_up(tiles_m * tiles_n, 8));
    const size_t ts = (size_t)npad * ldk;
    const __bf16* wt = reinterpret_cast<const __bf16*>(Wt);
#define DPC_SPLIT_LAUNCH(T, NTWV)                                                                                               \
    hipLaunchKernelGGL((contract_split_kernel<T, EPI, NTWV>), grid, dim3(256), 0, s, A, (long long)M, K, lda, wt, ldk, ts, N, C, ldc, \
                       (int)tiles_m, tiles_n, ep)
    if (terms == 2) { if (ntw == 4) DPC_SPLIT_LAUNCH(2, 4); else DPC_SPLIT_LAUNCH(2, 2); }
    else            DPC_SPLIT_LAUNCH(3, 2);
#undef DPC_SPLIT_LAUNCH
    DPC_HIP(hipGetLastError());
    return tiles_n;
}

bool split_shape_ok(const float* A, int K, int lda, const void* Wt, int terms, int N, int ldc)
{
    int ldk, npad;
    if (K < 1 || N < 1 || (terms != 2 && terms != 3)) return false;
    if (split_weights_elems(K, N, terms, &ldk, &npad) * 2 >= ((size_t)1 << 31) || (int64_t)lda * kBM * 4 >= ((int64_t)1 << 31)) return false;   // 32-bit buffer offsets
    return A && Wt && lda >= K && ldc >= N && lda % 4 == 0 && K % 4 == 0 && ldc % 4 == 0 && ldc <= npad && ((uintptr_t)A % 16) == 0 &&
           ((uintptr_t)Wt % 16) == 0;
}

}  // namespace

void launch_contract_split(const float* A, int64_t M, int K, int lda, const void* Wt, int terms, int N, float* C, int ldc,
                           hipStream_t s)
{
    DPC_REQUIRE(C && M >= 0 && split_shape_ok(A, K, lda, Wt, terms, N, ldc) && ((uintptr_t)C % 16) == 0, DPC_EINVAL,
                "contract_split: K, lda, ldc must be multiples of 4 (ldc within the column tiles of N), operands 16-byte aligned");
    if (M == 0) return;
    launch_split_kernel<0>(A, M, K, lda, Wt, terms, N, C, ldc, SplitEpi{}, 0, s);
}

int launch_contract_split_fused(const float* A, int64_t M, int K, int lda, const void* Wt, int terms, int N, float* C, int ldc,
                                const ContractEpilogue& e, hipStream_t s)
{
    DPC_REQUIRE(M >= 0 && split_shape_ok(A, K, lda, Wt, terms, N, ldc) && e.pk && e.part && (!e.store || (C && ((uintptr_t)C % 16) == 0)) &&
                    ((uintptr_t)e.pk % 16) == 0, DPC_EINVAL, "contract_split_fused: bad arguments");
    DPC_REQUIRE(e.ldpk >= ldc && e.R >= 32 && e.nsb >= 1 && (int64_t)e.nsb * e.R == M && e.part_stride >= M, DPC_EINVAL,
                "contract_split_fused: epilogue geometry does not match the rows");
    if (M == 0) return 0;
    return launch_split_kernel<1>(A, M, K, lda, Wt, terms, N, C, ldc,
                                  SplitEpi{reinterpret_cast<const float4*>(e.pk), e.ldpk, e.R, e.nsb, e.part, e.part_stride, e.store},
                                  e.max_slots, s);
}

}  // namespace dpc
