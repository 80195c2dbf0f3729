// fp32 MFMA contraction of a traverse iteration through an affine layer:
//   Cout[M, N] = A[M, K] * W[K, N]      (Matmul rewrite: the repeat / multiply / reduce of the
//                                        map semantics collapses into an inner product)
// M is huge (2 * batch * rows), K and N are layer widths.  gfx950, wave64,
// v_mfma_f32_32x32x2_f32 tiles.
//
// Tiling: a workgroup owns a BM x BN tile of Cout; each wavefront a WM x WN sub-tile held in
// accumulator registers as (WM/32) x (WN/32) MFMA tiles.  K advances in tiles of BK staged through
// double-buffered LDS (global -> registers -> LDS, one barrier per K tile).
//
// LDS layouts are chosen for the operand shape of the 32x32x2 MFMA (lane l feeds A[row l%32][k l/32]
// and B[k l/32][col l%32]):
//  * A tile is stored [BK/4][BM+1] float4 (k-quad major, one float4 of padding per plane): a lane
//    fetches the four consecutive k of its row with one 16-byte read, lanes of a half-wave read
//    consecutive float4.  Within each group of 8 k the lower half-wave takes k 0..3 and the upper
//    half k 4..7; MFMA step s of the group therefore multiplies k = {s, 4+s}.
//  * B tile is stored [BK][BN+8] floats.  A lane reads WN/32 consecutive floats of row k: element t
//    feeds MFMA column tile t, so column tile t owns the interleaved columns {(WN/32)*j + t}.  The
//    epilogue undoes the interleave for free: a lane ends up holding WN/32 consecutive output
//    columns per row and stores them with one vector store.
//
// Workgroup -> tile mapping is XCD aware: hardware deals workgroups round-robin to the 8 XCDs, so
// workgroup ids are re-linearised to give each XCD a contiguous run of tiles, N-tile index fastest;
// the tiles that re-read one A row panel then share one XCD's L2.
#include <type_traits>

#include "common.h"

namespace dpc {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Compile-time loop: indices reach the body as constants, so small per-thread arrays indexed by them stay
// in registers (a runtime-indexed array would be placed in scratch memory and serialise the prefetch).
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

template <int BM_, int BN_, int BK_, int WM_, int WN_, int MINW_ = 1>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_;
    static constexpr int MINW = MINW_;                          // wavefronts per SIMD the register budget must allow
    static constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN;
    static constexpr int THREADS = WAVES_M * WAVES_N * 64;
    static constexpr int MT = WM / 32, NT = WN / 32;            // MFMA tiles per wavefront
    static constexpr int A_PLANE = BM + 1;                      // float4 units
    static constexpr int A_STAGE = (BK / 4) * A_PLANE;          // float4 units
    static constexpr int B_ROW = BN + 8;                        // floats
    static constexpr int B_STAGE = BK * B_ROW;                  // floats
    static constexpr int A_LOADS = BM * BK / 4 / THREADS;       // float4 per thread per K tile
    static constexpr int B_LOADS = BK * BN / 4 / THREADS;
    static constexpr size_t LDS_BYTES = 2 * (size_t)A_STAGE * 16 + 2 * (size_t)B_STAGE * 4;
    static_assert(BM * BK / 4 % THREADS == 0 && BK * BN / 4 % THREADS == 0, "staging must divide evenly");
    static_assert(BK % 8 == 0 && WM % 32 == 0 && WN % 32 == 0 && NT <= 4, "tile shape");
};

// Fused epilogue (EPI = 1): the step that follows the contraction in the traversal is applied to the
// accumulators before they leave the registers.  For output element x of row m (group g = m / R, i.e.
// one side of one input) and column c, with packed parameters P = pk[g][c] = (pm, nm, kp, kn):
//     stored value  x * (x >= 0 ? pm : nm)           (sign-split ReLU step; skipped when store == 0)
//     row constant  += x * (x >= 0 ? kp : kn)        (nu and bias terms, or the box bound for the
//                                                     concretisation at the input layer)
// Row-constant partial sums are reduced over the tile's columns in a fixed order (butterfly over the
// 32 lanes of a half-wave, then over the workgroup's wave columns through LDS) and written to
// part[tile_n][m]; whoever consumes the constants adds the slots in index order, so results do not
// depend on scheduling.
struct EpiArgs {
    const float4* pk;
    int ldpk, R, nsb;
    float* part;
    long long part_stride;
    int store;
    int remap;          // 1: XCD-aware re-linearisation of workgroup ids
    // batched launches (gridDim.y problems of equal shape): element offsets per batch index of A, W and Cout
    long long strideA = 0, strideW = 0, strideC = 0;
};

template <class T, int EPI>
__global__ __launch_bounds__(T::THREADS, T::MINW) void contract_kernel(
    const float* __restrict__ A, int64_t M, int K, int lda, const float* __restrict__ W, int N, int ldw,
    float* __restrict__ Cout, int ldc, int tiles_m, int tiles_n, EpiArgs ep)
{
    extern __shared__ float4 lds[];
    float4* sA = lds;                                                        // [2][A_STAGE]
    float* sB = reinterpret_cast<float*>(lds + 2 * T::A_STAGE);              // [2][B_STAGE]
    if (gridDim.y > 1) {
        A += (long long)blockIdx.y * ep.strideA;
        W += (long long)blockIdx.y * ep.strideW;
        Cout += (long long)blockIdx.y * ep.strideC;
    }

    // XCD-aware re-linearisation (gridDim.x is a multiple of 8)
    const int per_xcd = gridDim.x >> 3;
    const int v = ep.remap ? (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3) : blockIdx.x;
    if (v >= tiles_m * tiles_n) return;
    const int tm = v / tiles_n, tn = v - tm * tiles_n;
    const int64_t m0 = (int64_t)tm * T::BM;
    const int n0 = tn * T::BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wrow0 = (wave / T::WAVES_N) * T::WM, wcol0 = (wave % T::WAVES_N) * T::WN;
    const int l32 = lane & 31, kq = lane >> 5;

    const int K4 = (K + 3) & ~3, N4 = (N + 3) & ~3;
    const int nk = (K + T::BK - 1) / T::BK;
    const bool wave_active = n0 + wcol0 < N4;

    // Per-thread staging slots.  Each slot is a set of scalar variables (not an array): the prefetched
    // tile must live in registers across the MFMA section, and arrays captured by the helper lambdas were
    // being placed in scratch memory by the compiler, which serialised every prefetch.
    struct Slot { const float* ptr; int k; int lds; bool ok; };
    auto a_slot = [&](int i) __attribute__((always_inline)) {
        const int idx = tid + T::THREADS * i;
        const int row = idx / (T::BK / 4), kc = idx % (T::BK / 4);
        int64_t gr = m0 + row;
        if (gr > M - 1) gr = M - 1;                     // clamp: rows past M are computed, never stored
        return Slot{A + gr * lda + kc * 4, kc * 4, kc * T::A_PLANE + row, true};
    };
    auto b_slot = [&](int i) __attribute__((always_inline)) {
        const int idx = tid + T::THREADS * i;
        const int kr = idx / (T::BN / 4), nc = idx % (T::BN / 4);
        return Slot{W + (size_t)kr * ldw + n0 + nc * 4, kr, kr * T::B_ROW + nc * 4, n0 + nc * 4 < N4};
    };
    static_assert(T::A_LOADS <= 4 && T::B_LOADS <= 4, "at most four staging slots per operand");
    const Slot sa0 = a_slot(0), sa1 = a_slot(T::A_LOADS > 1 ? 1 : 0), sa2 = a_slot(T::A_LOADS > 2 ? 2 : 0),
               sa3 = a_slot(T::A_LOADS > 3 ? 3 : 0);
    const Slot sb0 = b_slot(0), sb1 = b_slot(T::B_LOADS > 1 ? 1 : 0), sb2 = b_slot(T::B_LOADS > 2 ? 2 : 0),
               sb3 = b_slot(T::B_LOADS > 3 ? 3 : 0);

    floatx16 acc[T::MT][T::NT];
#pragma unroll
    for (int i = 0; i < T::MT; ++i)
#pragma unroll
        for (int j = 0; j < T::NT; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    typedef float vf4 __attribute__((ext_vector_type(4)));
    vf4 ra0 = {0, 0, 0, 0}, ra1 = ra0, ra2 = ra0, ra3 = ra0, rb0 = ra0, rb1 = ra0, rb2 = ra0, rb3 = ra0;
    const vf4 zero4 = {0.f, 0.f, 0.f, 0.f};

#define DPC_LOAD_A(S, R) R = (k0 + S.k < K4) ? *reinterpret_cast<const vf4*>(S.ptr + k0) : zero4
#define DPC_LOAD_B(S, R) R = (S.ok && k0 + S.k < K) ? *reinterpret_cast<const vf4*>(S.ptr + (size_t)k0 * ldw) : zero4
    auto load_tile = [&](int kt) __attribute__((always_inline)) {
        const int k0 = kt * T::BK;
        DPC_LOAD_A(sa0, ra0);
        if constexpr (T::A_LOADS > 1) DPC_LOAD_A(sa1, ra1);
        if constexpr (T::A_LOADS > 2) DPC_LOAD_A(sa2, ra2);
        if constexpr (T::A_LOADS > 3) DPC_LOAD_A(sa3, ra3);
        DPC_LOAD_B(sb0, rb0);
        if constexpr (T::B_LOADS > 1) DPC_LOAD_B(sb1, rb1);
        if constexpr (T::B_LOADS > 2) DPC_LOAD_B(sb2, rb2);
        if constexpr (T::B_LOADS > 3) DPC_LOAD_B(sb3, rb3);
    };
#undef DPC_LOAD_A
#undef DPC_LOAD_B
    auto store_tile = [&](int stage) __attribute__((always_inline)) {
        vf4* dA = reinterpret_cast<vf4*>(sA + stage * T::A_STAGE);
        float* dB = sB + stage * T::B_STAGE;
        dA[sa0.lds] = ra0;
        if constexpr (T::A_LOADS > 1) dA[sa1.lds] = ra1;
        if constexpr (T::A_LOADS > 2) dA[sa2.lds] = ra2;
        if constexpr (T::A_LOADS > 3) dA[sa3.lds] = ra3;
        *reinterpret_cast<vf4*>(dB + sb0.lds) = rb0;
        if constexpr (T::B_LOADS > 1) *reinterpret_cast<vf4*>(dB + sb1.lds) = rb1;
        if constexpr (T::B_LOADS > 2) *reinterpret_cast<vf4*>(dB + sb2.lds) = rb2;
        if constexpr (T::B_LOADS > 3) *reinterpret_cast<vf4*>(dB + sb3.lds) = rb3;
    };

    load_tile(0);
    store_tile(0);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int stage = kt & 1;
        if (kt + 1 < nk) load_tile(kt + 1);

        const float4* pa = sA + stage * T::A_STAGE + wrow0 + l32;
        const float* pb = sB + stage * T::B_STAGE + wcol0 + T::NT * l32;
        if (wave_active)                 // a wavefront whose columns all lie past N only helps staging
#pragma unroll
        for (int g = 0; g < T::BK / 8; ++g) {
            float4 a[T::MT];
#pragma unroll
            for (int mt = 0; mt < T::MT; ++mt) a[mt] = pa[(2 * g + kq) * T::A_PLANE + mt * 32];
            float b[4][T::NT];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const float* p = pb + (8 * g + 4 * kq + s) * T::B_ROW;
                if constexpr (T::NT == 1) {
                    b[s][0] = p[0];
                } else if constexpr (T::NT == 2) {
                    const float2 t = *reinterpret_cast<const float2*>(p);
                    b[s][0] = t.x; b[s][1] = t.y;
                } else {
                    const float4 t = *reinterpret_cast<const float4*>(p);
                    b[s][0] = t.x; b[s][1] = t.y; b[s][2] = t.z;
                    if constexpr (T::NT == 4) b[s][3] = t.w;
                }
            }
#pragma unroll
            for (int s = 0; s < 4; ++s) {
#pragma unroll
                for (int mt = 0; mt < T::MT; ++mt) {
                    const float av = s == 0 ? a[mt].x : s == 1 ? a[mt].y : s == 2 ? a[mt].z : a[mt].w;
#pragma unroll
                    for (int nt = 0; nt < T::NT; ++nt)
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, b[s][nt], acc[mt][nt], 0, 0, 0);
                }
            }
        }

        if (kt + 1 < nk) store_tile(stage ^ 1);
        __syncthreads();
    }

    if constexpr (EPI == 1) {
        float* sRow = reinterpret_cast<float*>(lds);              // [WAVES_N][BM], the K loop is done with LDS
        const int wn = wave % T::WAVES_N;
        const float4 zero4e = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int mt = 0; mt < T::MT; ++mt) {
            const int64_t rb = m0 + wrow0 + mt * 32;
            const int64_t rclamp = rb < M ? rb : M - 1;
            const int g_lo = (int)(rclamp / ep.R);
            const int64_t boundary = (int64_t)(g_lo + 1) * ep.R;          // first row of the next group
            const bool split = boundary < rb + 32;                         // wave-uniform; R >= 32: at most one
            const int g_hi = g_lo + 1 < ep.nsb ? g_lo + 1 : ep.nsb - 1;
            const int col = n0 + wcol0 + T::NT * l32;
            float4 pa[T::NT], pb[T::NT];
#pragma unroll
            for (int nt = 0; nt < T::NT; ++nt) {
                const bool ok = col + nt < ep.ldpk;
                pa[nt] = ok ? ep.pk[(size_t)g_lo * ep.ldpk + col + nt] : zero4e;
                pb[nt] = (ok && split) ? ep.pk[(size_t)g_hi * ep.ldpk + col + nt] : pa[nt];
            }
            float rs[16];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int64_t row = rb + 8 * i + 4 * kq + j;
                    const bool useb = row >= boundary;
                    float o[T::NT];
                    float sum = 0.0f;
#pragma unroll
                    for (int nt = 0; nt < T::NT; ++nt) {
                        const float x = acc[mt][nt][4 * i + j];
                        const float4 P = useb ? pb[nt] : pa[nt];
                        const bool pos = x >= 0.0f;
                        o[nt] = x * (pos ? P.x : P.y);
                        sum += x * (pos ? P.z : P.w);
                    }
                    rs[4 * i + j] = sum;
                    if (ep.store && row < M && col < ldc) {
                        float* dst = Cout + row * ldc + col;
                        if constexpr (T::NT == 1) {
                            dst[0] = o[0];
                        } else if constexpr (T::NT == 2) {
                            *reinterpret_cast<float2*>(dst) = make_float2(o[0], o[1]);
                        } else if constexpr (T::NT == 4) {
                            *reinterpret_cast<float4*>(dst) = make_float4(o[0], o[1], o[2], o[3]);
                        } else {
#pragma unroll
                            for (int nt = 0; nt < T::NT; ++nt)
                                if (col + nt < ldc) dst[nt] = o[nt];
                        }
                    }
                }
            }
            // Butterfly with halving over the 32 lanes that share these rows: after the steps with lane
            // bits 0..3 a lane holds the sum over its 16-lane group of register index 8*b0+4*b1+2*b2+b3,
            // the last step adds the two groups.
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
                const int v = 8 * (l32 & 1) + 4 * ((l32 >> 1) & 1) + 2 * ((l32 >> 2) & 1) + ((l32 >> 3) & 1);
                sRow[wn * T::BM + wrow0 + mt * 32 + 8 * (v >> 2) + 4 * kq + (v & 3)] = v1;
            }
        }
        __syncthreads();
        for (int r = tid; r < T::BM; r += T::THREADS) {
            float t = 0.0f;
#pragma unroll
            for (int w = 0; w < T::WAVES_N; ++w) t += sRow[w * T::BM + r];
            if (m0 + r < M) ep.part[(size_t)tn * ep.part_stride + m0 + r] = t;
        }
        return;
    }

    // epilogue: accumulator register e = 4*i + j of a lane is row 8*i + 4*(lane/32) + j, column lane%32
    // of its MFMA tile; column tile nt owns interleaved columns NT*l32 + nt.
#pragma unroll
    for (int mt = 0; mt < T::MT; ++mt) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t row = m0 + wrow0 + mt * 32 + 8 * i + 4 * kq + j;
                const int col = n0 + wcol0 + T::NT * l32;
                if (row >= M || col >= ldc) continue;
                float o[T::NT];
#pragma unroll
                for (int nt = 0; nt < T::NT; ++nt) o[nt] = (col + nt < N) ? acc[mt][nt][4 * i + j] : 0.0f;
                float* dst = Cout + row * ldc + col;
                if constexpr (T::NT == 1) {
                    dst[0] = o[0];
                } else if constexpr (T::NT == 2) {
                    *reinterpret_cast<float2*>(dst) = make_float2(o[0], o[1]);
                } else if constexpr (T::NT == 4) {
                    *reinterpret_cast<float4*>(dst) = make_float4(o[0], o[1], o[2], o[3]);
                } else {
#pragma unroll
                    for (int nt = 0; nt < T::NT; ++nt)
                        if (col + nt < ldc) dst[nt] = o[nt];
                }
            }
        }
    }
}

template <class T, int EPI>
int launch_variant(const float* A, int64_t M, int K, int lda, const float* W, int N, int ldw, float* Cout,
                   int ldc, const EpiArgs& ep, int max_slots, hipStream_t s, int batches = 1)
{
    ensure_dynamic_lds(reinterpret_cast<const void*>(&contract_kernel<T, EPI>), (int)T::LDS_BYTES);
    static_assert(EPI == 0 || T::LDS_BYTES >= (size_t)T::WAVES_N * T::BM * 4, "row sums must fit the K-loop LDS");
    const int64_t tiles_m = ceil_div(M, T::BM);
    const int tiles_n = (int)ceil_div(ldc, T::BN);          // padding columns of Cout are written too
    const int64_t tiles = tiles_m * tiles_n;
    DPC_REQUIRE(tiles_m < (1 << 30) && tiles < (int64_t)1 << 31, DPC_EINVAL, "contract: too many tiles");
    if (EPI == 1 && tiles_n > max_slots) return -1;
    const unsigned grid = (unsigned)round_up(tiles, 8);
    hipLaunchKernelGGL((contract_kernel<T, EPI>), dim3(grid, (unsigned)batches), dim3(T::THREADS), T::LDS_BYTES, s, A, M, K,
                       lda, W, N, ldw, Cout, ldc, (int)tiles_m, tiles_n, ep);
    DPC_HIP(hipGetLastError());
    return tiles_n;
}


// Tile choice from the problem shape (measured on cfg2- and cfg5-sized contractions):
//  * fewer than 512 tiles of 128x128: 64x64 tiles, so that the grid still covers the 256 CUs;
//  * otherwise 128x256 tiles (8 wavefronts of 64x64, K tile 16), unless the last 256-wide column tile
//    would be at most half used (e.g. 784 columns), where 128x128 tiles waste less.
int pick_variant(int64_t M, int ldc, int K)
{
    const int64_t tiles128 = ceil_div(M, 128) * ceil_div(ldc, 128);
    // small problems are bound by the latency of their K loop: fewer, longer K steps (64 x 64 tiles, 64 or 32 deep)
    if (tiles128 < 512) return K >= 256 ? 18 : K >= 64 ? 19 : 9;
    const int rem = ldc % 256;
    return (rem != 0 && rem <= 128) ? 17 : 7;
}

}  // namespace


void launch_contract(const float* A, int64_t M, int K, int lda, const float* W, int N, int ldw,
                     float* Cout, int ldc, hipStream_t s)
{
    DPC_REQUIRE(A && W && Cout && M >= 0 && K >= 1 && N >= 1, DPC_EINVAL, "contract: bad arguments");
    DPC_REQUIRE(lda >= K && ldw >= N && ldc >= N && lda % 4 == 0 && ldw % 4 == 0 && ldc % 4 == 0, DPC_EINVAL,
                "contract: leading dimensions must cover the matrix and be multiples of 4");
    DPC_REQUIRE(((uintptr_t)A % 16) == 0 && ((uintptr_t)W % 16) == 0 && ((uintptr_t)Cout % 16) == 0, DPC_EINVAL,
                "contract: buffers must be 16-byte aligned");
    if (M == 0) return;
    const int variant = tune(TK_CONTRACT_VARIANT) >= 0 ? tune(TK_CONTRACT_VARIANT) : pick_variant(M, ldc, K);
    switch (variant) {
        case 1:  launch_variant<Tile<256, 128, 16, 64, 64>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 2:  launch_variant<Tile<128, 128, 16, 64, 64>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 3:  launch_variant<Tile<256, 128, 16, 128, 64>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 4:  launch_variant<Tile<128, 256, 16, 64, 128>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 5:  launch_variant<Tile<256, 128, 32, 64, 64>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 6:  launch_variant<Tile<256, 256, 16, 128, 64>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 7:  launch_variant<Tile<128, 256, 16, 64, 64>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 8:  launch_variant<Tile<64, 128, 16, 32, 64>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 9:  launch_variant<Tile<64, 64, 16, 32, 32>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 10: launch_variant<Tile<128, 128, 8, 64, 64, 3>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 16: launch_variant<Tile<128, 128, 8, 64, 64, 4>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 17: launch_variant<Tile<128, 128, 16, 64, 64, 3>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 18: launch_variant<Tile<64, 64, 64, 32, 32>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 19: launch_variant<Tile<64, 64, 32, 32, 32>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 20: launch_variant<Tile<32, 64, 32, 32, 32>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 11: launch_variant<Tile<64, 64, 8, 32, 64>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 12: launch_variant<Tile<128, 64, 16, 64, 32>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 13: launch_variant<Tile<64, 128, 8, 64, 64>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 14: launch_variant<Tile<128, 128, 8, 128, 64>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        case 15: launch_variant<Tile<256, 128, 8, 128, 64>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
        default: launch_variant<Tile<128, 128, 32, 64, 64>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, EpiArgs{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP)}, 0, s); break;
    }
}


void launch_contract_batched(const float* A, int64_t strideA, int64_t M, int K, int lda, const float* W, int64_t strideW, int N,
                             int ldw, float* Cout, int64_t strideC, int ldc, int batches, hipStream_t s)
{
    DPC_REQUIRE(A && W && Cout && M >= 0 && K >= 1 && N >= 1 && batches >= 0 && batches <= 65535, DPC_EINVAL,
                "contract_batched: bad arguments");
    DPC_REQUIRE(lda >= K && ldw >= N && ldc >= N && lda % 4 == 0 && ldw % 4 == 0 && ldc % 4 == 0 && strideA % 4 == 0 &&
                    strideW % 4 == 0 && strideC % 4 == 0, DPC_EINVAL,
                "contract_batched: leading dimensions and batch strides must cover the matrix and be multiples of 4");
    DPC_REQUIRE(((uintptr_t)A % 16) == 0 && ((uintptr_t)W % 16) == 0 && ((uintptr_t)Cout % 16) == 0, DPC_EINVAL,
                "contract_batched: buffers must be 16-byte aligned");
    if (M == 0 || batches == 0) return;
    EpiArgs ep{nullptr, 0, 0, 0, nullptr, 0, 0, tune(TK_CONTRACT_REMAP), (long long)strideA, (long long)strideW, (long long)strideC};
    // tile choice as for one problem of batches * M rows; problems of at most 512 rows tile better with 64x64
    // (measured on the 500-row steps of ReuseCert)
    const int variant = tune(TK_CONTRACT_VARIANT) >= 0 ? tune(TK_CONTRACT_VARIANT) : M <= 512 ? 9 : pick_variant(M * batches, ldc, 0);
    switch (variant) {
        case 7:  launch_variant<Tile<128, 256, 16, 64, 64>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, ep, 0, s, batches); break;
        case 17: launch_variant<Tile<128, 128, 16, 64, 64, 3>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, ep, 0, s, batches); break;
        default: launch_variant<Tile<64, 64, 16, 32, 32>, 0>(A, M, K, lda, W, N, ldw, Cout, ldc, ep, 0, s, batches); break;
    }
}

int launch_contract_fused(const float* A, int64_t M, int K, int lda, const float* W, int N, int ldw,
                          float* Cout, int ldc, const ContractEpilogue& e, hipStream_t s)
{
    DPC_REQUIRE(A && W && M >= 0 && K >= 1 && N >= 1 && e.pk && e.part, DPC_EINVAL, "contract_fused: bad arguments");
    DPC_REQUIRE(!e.store || Cout, DPC_EINVAL, "contract_fused: output missing");
    DPC_REQUIRE(lda >= K && ldw >= N && ldc >= N && lda % 4 == 0 && ldw % 4 == 0 && ldc % 4 == 0, DPC_EINVAL,
                "contract_fused: leading dimensions must cover the matrix and be multiples of 4");
    DPC_REQUIRE(((uintptr_t)A % 16) == 0 && ((uintptr_t)W % 16) == 0 && ((uintptr_t)Cout % 16) == 0 &&
                    ((uintptr_t)e.pk % 16) == 0, DPC_EINVAL, "contract_fused: buffers must be 16-byte aligned");
    DPC_REQUIRE(e.ldpk >= ldc && e.R >= 32 && e.nsb >= 1 && (int64_t)e.nsb * e.R == M && e.part_stride >= M, DPC_EINVAL,
                "contract_fused: epilogue geometry does not match the rows");
    if (M == 0) return 0;
    const int variant = tune(TK_CONTRACT_VARIANT) >= 0 ? tune(TK_CONTRACT_VARIANT) : pick_variant(M, ldc, K);
    EpiArgs ep{reinterpret_cast<const float4*>(e.pk), e.ldpk, e.R, e.nsb, e.part, e.part_stride, e.store, tune(TK_CONTRACT_REMAP)};
    switch (variant) {      // the fused epilogue is instantiated for the tiles the shape heuristic can pick
        case 17: return launch_variant<Tile<128, 128, 16, 64, 64, 3>, 1>(A, M, K, lda, W, N, ldw, Cout, ldc, ep, e.max_slots, s);
        case 7:  return launch_variant<Tile<128, 256, 16, 64, 64>, 1>(A, M, K, lda, W, N, ldw, Cout, ldc, ep, e.max_slots, s);
        case 9:  return launch_variant<Tile<64, 64, 16, 32, 32>, 1>(A, M, K, lda, W, N, ldw, Cout, ldc, ep, e.max_slots, s);
        case 10: return launch_variant<Tile<128, 128, 8, 64, 64, 3>, 1>(A, M, K, lda, W, N, ldw, Cout, ldc, ep, e.max_slots, s);
        case 19: return launch_variant<Tile<64, 64, 32, 32, 32>, 1>(A, M, K, lda, W, N, ldw, Cout, ldc, ep, e.max_slots, s);
        case 18: return launch_variant<Tile<64, 64, 64, 32, 32>, 1>(A, M, K, lda, W, N, ldw, Cout, ldc, ep, e.max_slots, s);
        default: return -1;
    }
}

}  // namespace dpc
