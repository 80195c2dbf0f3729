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
#include "common.h"

namespace dpc {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

template <int BM_, int BN_, int BK_, int WM_, int WN_>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_;
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

template <class T>
__global__ __launch_bounds__(T::THREADS) void contract_kernel(
    const float* __restrict__ A, int64_t M, int K, int lda, const float* __restrict__ W, int N, int ldw,
    float* __restrict__ Cout, int ldc, int tiles_m, int tiles_n)
{
    extern __shared__ float4 lds[];
    float4* sA = lds;                                                        // [2][A_STAGE]
    float* sB = reinterpret_cast<float*>(lds + 2 * T::A_STAGE);              // [2][B_STAGE]

    // XCD-aware re-linearisation (gridDim.x is a multiple of 8)
    const int per_xcd = gridDim.x >> 3;
    const int v = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (v >= tiles_m * tiles_n) return;
    const int tm = v / tiles_n, tn = v - tm * tiles_n;
    const int64_t m0 = (int64_t)tm * T::BM;
    const int n0 = tn * T::BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wrow0 = (wave / T::WAVES_N) * T::WM, wcol0 = (wave % T::WAVES_N) * T::WN;
    const int l32 = lane & 31, kq = lane >> 5;

    const int K4 = (K + 3) & ~3, N4 = (N + 3) & ~3;
    const int nk = (K + T::BK - 1) / T::BK;

    // per-thread staging coordinates
    const float* a_ptr[T::A_LOADS];
    int a_kc[T::A_LOADS], a_lds[T::A_LOADS];
#pragma unroll
    for (int i = 0; i < T::A_LOADS; ++i) {
        const int idx = tid + T::THREADS * i;
        const int row = idx / (T::BK / 4), kc = idx % (T::BK / 4);
        int64_t gr = m0 + row;
        if (gr > M - 1) gr = M - 1;                     // clamp: rows past M are computed, never stored
        a_ptr[i] = A + gr * lda + kc * 4;
        a_kc[i] = kc * 4;
        a_lds[i] = kc * T::A_PLANE + row;
    }
    const float* b_ptr[T::B_LOADS];
    int b_kr[T::B_LOADS], b_lds[T::B_LOADS];
    bool b_ok[T::B_LOADS];
#pragma unroll
    for (int i = 0; i < T::B_LOADS; ++i) {
        const int idx = tid + T::THREADS * i;
        const int kr = idx / (T::BN / 4), nc = idx % (T::BN / 4);
        b_ptr[i] = W + (size_t)kr * ldw + n0 + nc * 4;
        b_kr[i] = kr;
        b_ok[i] = n0 + nc * 4 < N4;
        b_lds[i] = kr * T::B_ROW + nc * 4;
    }

    floatx16 acc[T::MT][T::NT];
#pragma unroll
    for (int i = 0; i < T::MT; ++i)
#pragma unroll
        for (int j = 0; j < T::NT; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    float4 ra[T::A_LOADS], rb[T::B_LOADS];
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);

    auto load_tile = [&](int kt) {
        const int k0 = kt * T::BK;
#pragma unroll
        for (int i = 0; i < T::A_LOADS; ++i)
            ra[i] = (k0 + a_kc[i] < K4) ? *reinterpret_cast<const float4*>(a_ptr[i] + k0) : zero4;
#pragma unroll
        for (int i = 0; i < T::B_LOADS; ++i)
            rb[i] = (b_ok[i] && k0 + b_kr[i] < K)
                        ? *reinterpret_cast<const float4*>(b_ptr[i] + (size_t)k0 * ldw) : zero4;
    };
    auto store_tile = [&](int stage) {
#pragma unroll
        for (int i = 0; i < T::A_LOADS; ++i) sA[stage * T::A_STAGE + a_lds[i]] = ra[i];
#pragma unroll
        for (int i = 0; i < T::B_LOADS; ++i)
            *reinterpret_cast<float4*>(sB + stage * T::B_STAGE + b_lds[i]) = rb[i];
    };

    load_tile(0);
    store_tile(0);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int stage = kt & 1;
        if (kt + 1 < nk) load_tile(kt + 1);

        const float4* pa = sA + stage * T::A_STAGE + wrow0 + l32;
        const float* pb = sB + stage * T::B_STAGE + wcol0 + T::NT * l32;
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

template <class T>
void launch_variant(const float* A, int64_t M, int K, int lda, const float* W, int N, int ldw, float* Cout,
                    int ldc, hipStream_t s)
{
    static bool configured = false;
    if (!configured) {
        DPC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&contract_kernel<T>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)T::LDS_BYTES));
        configured = true;
    }
    const int64_t tiles_m = ceil_div(M, T::BM);
    const int tiles_n = (int)ceil_div(ldc, T::BN);          // padding columns of Cout are written too
    const int64_t tiles = tiles_m * tiles_n;
    DPC_REQUIRE(tiles_m < (1 << 30) && tiles < (int64_t)1 << 31, DPC_EINVAL, "contract: too many tiles");
    const unsigned grid = (unsigned)round_up(tiles, 8);
    hipLaunchKernelGGL(contract_kernel<T>, dim3(grid), dim3(T::THREADS), T::LDS_BYTES, s, A, M, K, lda, W, N, ldw,
                       Cout, ldc, (int)tiles_m, tiles_n);
    DPC_HIP(hipGetLastError());
}

int g_variant = -1;      // -1: chosen from the problem shape

}  // namespace

void set_contract_variant(int v) { g_variant = v; }

void launch_contract(const float* A, int64_t M, int K, int lda, const float* W, int N, int ldw,
                     float* Cout, int ldc, hipStream_t s)
{
    DPC_REQUIRE(A && W && Cout && M >= 0 && K >= 1 && N >= 1, DPC_EINVAL, "contract: bad arguments");
    DPC_REQUIRE(lda >= K && ldw >= N && ldc >= N && lda % 4 == 0 && ldw % 4 == 0 && ldc % 4 == 0, DPC_EINVAL,
                "contract: leading dimensions must cover the matrix and be multiples of 4");
    DPC_REQUIRE(((uintptr_t)A % 16) == 0 && ((uintptr_t)W % 16) == 0 && ((uintptr_t)Cout % 16) == 0, DPC_EINVAL,
                "contract: buffers must be 16-byte aligned");
    if (M == 0) return;
    int variant = g_variant;
    if (variant < 0) {
        // Large problems: 128x128 tiles with a short K tile (small LDS footprint -> three workgroups per
        // CU hide each other's barrier and load latency).  Small problems: 64x64 tiles so that the grid
        // still covers the 256 CUs.
        const int64_t tiles128 = ceil_div(M, 128) * ceil_div(ldc, 128);
        variant = tiles128 >= 512 ? 10 : 9;
    }
    switch (variant) {
        case 1:  launch_variant<Tile<256, 128, 16, 64, 64>>(A, M, K, lda, W, N, ldw, Cout, ldc, s); break;
        case 2:  launch_variant<Tile<128, 128, 16, 64, 64>>(A, M, K, lda, W, N, ldw, Cout, ldc, s); break;
        case 3:  launch_variant<Tile<256, 128, 16, 128, 64>>(A, M, K, lda, W, N, ldw, Cout, ldc, s); break;
        case 4:  launch_variant<Tile<128, 256, 16, 64, 128>>(A, M, K, lda, W, N, ldw, Cout, ldc, s); break;
        case 5:  launch_variant<Tile<256, 128, 32, 64, 64>>(A, M, K, lda, W, N, ldw, Cout, ldc, s); break;
        case 6:  launch_variant<Tile<256, 256, 16, 128, 64>>(A, M, K, lda, W, N, ldw, Cout, ldc, s); break;
        case 7:  launch_variant<Tile<128, 256, 16, 64, 64>>(A, M, K, lda, W, N, ldw, Cout, ldc, s); break;
        case 8:  launch_variant<Tile<64, 128, 16, 32, 64>>(A, M, K, lda, W, N, ldw, Cout, ldc, s); break;
        case 9:  launch_variant<Tile<64, 64, 16, 32, 32>>(A, M, K, lda, W, N, ldw, Cout, ldc, s); break;
        case 10: launch_variant<Tile<128, 128, 8, 64, 64>>(A, M, K, lda, W, N, ldw, Cout, ldc, s); break;
        case 11: launch_variant<Tile<64, 64, 8, 32, 64>>(A, M, K, lda, W, N, ldw, Cout, ldc, s); break;
        case 12: launch_variant<Tile<128, 64, 16, 64, 32>>(A, M, K, lda, W, N, ldw, Cout, ldc, s); break;
        case 13: launch_variant<Tile<64, 128, 8, 64, 64>>(A, M, K, lda, W, N, ldw, Cout, ldc, s); break;
        case 14: launch_variant<Tile<128, 128, 8, 128, 64>>(A, M, K, lda, W, N, ldw, Cout, ldc, s); break;
        case 15: launch_variant<Tile<256, 128, 8, 128, 64>>(A, M, K, lda, W, N, ldw, Cout, ldc, s); break;
        default: launch_variant<Tile<128, 128, 32, 64, 64>>(A, M, K, lda, W, N, ldw, Cout, ldc, s); break;
    }
}

}  // namespace dpc
