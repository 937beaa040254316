// C = A * B, bfloat16 operands, fp32 accumulation on the matrix cores
// (v_mfma_f32_32x32x16_bf16), bfloat16 result.  A is row-major M x K; B is
// stored N x K with K contiguous (b_is_nk) -- both operands are then read as
// 16-byte runs along K -- or row-major K x N (handled by the generic kernel).
// Tiles of A and B are staged through LDS; every global tile load and every
// store of C carries the fence on its final address.  LDS is not fenced.
#include "launchers.hpp"

namespace gd {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ uint32_t gemm_f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// ---- generic kernel: any shape, any alignment, either layout of B -------------------
// One thread per entry of C, 2-byte accesses, fp32 accumulation in k order.
template <int V>
__global__ __launch_bounds__(256) void k_gemm_generic(gd_args_gemm p, FenceArgs fa)
{
    const Fence<V> F(fa);
    const uint64_t total = (uint64_t)p.M * p.N;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t e = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
        const uint64_t m = e / p.N, n = e % p.N;
        float acc = 0.0f;
        for (uint64_t k = 0; k < p.K; ++k) {
            const uint32_t ha = F.template ld<uint16_t>(p.A + 2 * (m * p.K + k));
            const uint32_t hb = F.template ld<uint16_t>(p.B + 2 * (p.b_is_nk ? n * p.K + k : k * p.N + n));
            acc += __uint_as_float(ha << 16) * __uint_as_float(hb << 16);
        }
        F.template st<uint16_t>(p.C + 2 * e, (uint16_t)gemm_f32_to_bf16(acc));
    }
}

// ---- tiled MFMA kernel: B stored N x K, K % 8 == 0, 16-byte aligned pointers ----------
// Workgroup tile BM x BN, K step BK, WM x WN wavefronts; each wavefront owns a
// (BM/WM) x (BN/WN) block of C made of 32x32 MFMA tiles.
template <int V, int BM, int BN, int BK, int WM, int WN>
__global__ __launch_bounds__(WM *WN * 64) void k_gemm_nk(gd_args_gemm p, FenceArgs fa)
{
    constexpr int NT = WM * WN * 64;
    constexpr int GPR = BK / 8;                 // 16-byte granules per tile row
    constexpr int LDS_ROW = BK + 8;             // padded row, in bf16 elements
    constexpr int A_LOADS = BM * GPR / NT;
    constexpr int B_LOADS = BN * GPR / NT;
    constexpr int TM = BM / WM / 32;
    constexpr int TN = BN / WN / 32;
    static_assert(BM * GPR % NT == 0 && BN * GPR % NT == 0, "tile loads must divide evenly");

    const Fence<V> F(fa);
    __shared__ __attribute__((aligned(16))) uint16_t As[BM * LDS_ROW];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[BN * LDS_ROW];

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63, wave = tid >> 6;
    const uint32_t wm = wave / WN, wn = wave % WN;
    const uint32_t tiles_n = (p.N + BN - 1) / BN;
    const uint32_t m0 = (blockIdx.x / tiles_n) * BM;
    const uint32_t n0 = (blockIdx.x % tiles_n) * BN;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    u32x4 ra[A_LOADS], rb[B_LOADS];
    auto load_tile = [&](uint32_t k0) {
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) {
            const uint32_t q = tid + i * NT, row = q / GPR, g = q % GPR;
            const uint32_t m = m0 + row, k = k0 + g * 8;
            ra[i] = (u32x4){0, 0, 0, 0};
            if (m < p.M && k < p.K) ra[i] = F.template ld<u32x4>(p.A + 2 * ((uint64_t)m * p.K + k));
        }
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i) {
            const uint32_t q = tid + i * NT, row = q / GPR, g = q % GPR;
            const uint32_t n = n0 + row, k = k0 + g * 8;
            rb[i] = (u32x4){0, 0, 0, 0};
            if (n < p.N && k < p.K) rb[i] = F.template ld<u32x4>(p.B + 2 * ((uint64_t)n * p.K + k));
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) {
            const uint32_t q = tid + i * NT, row = q / GPR, g = q % GPR;
            *(u32x4 *)&As[row * LDS_ROW + g * 8] = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i) {
            const uint32_t q = tid + i * NT, row = q / GPR, g = q % GPR;
            *(u32x4 *)&Bs[row * LDS_ROW + g * 8] = rb[i];
        }
    };

    load_tile(0);
    for (uint32_t k0 = 0; k0 < p.K; k0 += BK) {
        store_tile();
        __syncthreads();
        if (k0 + BK < p.K) load_tile(k0 + BK);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 fa_[TM], fb_[TN];
            const uint32_t kcol = kk * 16 + (lane >> 5) * 8;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const uint32_t row = wm * (BM / WM) + i * 32 + (lane & 31);
                fa_[i] = __builtin_bit_cast(bf16x8, *(const u32x4 *)&As[row * LDS_ROW + kcol]);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const uint32_t row = wn * (BN / WN) + j * 32 + (lane & 31);
                fb_[j] = __builtin_bit_cast(bf16x8, *(const u32x4 *)&Bs[row * LDS_ROW + kcol]);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa_[i], fb_[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // acc[i][j][r] is C[row, col] with row = 8*(r/4) + 4*(lane/32) + r%4, col = lane%32
    // inside the 32x32 tile.
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const uint32_t m = m0 + wm * (BM / WM) + i * 32 + 8 * (r / 4) + 4 * (lane >> 5) + (r & 3);
                const uint32_t n = n0 + wn * (BN / WN) + j * 32 + (lane & 31);
                if (m < p.M && n < p.N)
                    F.template st<uint16_t>(p.C + 2 * ((uint64_t)m * p.N + n),
                                            (uint16_t)gemm_f32_to_bf16(acc[i][j][r]));
            }
}

// ---- launcher ---------------------------------------------------------------------------

int launch_gemm_bf16(const void *args, const FenceArgs &f, int variant, const Shape &shape,
                     hipStream_t stream)
{
    const gd_args_gemm &p = *(const gd_args_gemm *)args;
    if (shape.grid || shape.block) return GD_EINVAL;
    if (p.M == 0 || p.N == 0) return GD_OK;
    const bool tiled = p.b_is_nk && p.K > 0 && (p.K % 8) == 0 && ((p.A | p.B) & 15) == 0;
    if (tiled) {
        constexpr int BM = 128, BN = 128, BK = 32;
        const uint64_t tiles = (uint64_t)((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN);
        if (tiles > 0x7fffffffull) return GD_ESHAPE;
#define K_GEMM_NK(V) k_gemm_nk<V, BM, BN, BK, 2, 2>
        switch (variant) {
        case V_NONE:  hipLaunchKernelGGL((K_GEMM_NK(V_NONE)), dim3((uint32_t)tiles), dim3(256), 0, stream, p, f); break;
        case V_BIT32: hipLaunchKernelGGL((K_GEMM_NK(V_BIT32)), dim3((uint32_t)tiles), dim3(256), 0, stream, p, f); break;
        case V_BIT64: hipLaunchKernelGGL((K_GEMM_NK(V_BIT64)), dim3((uint32_t)tiles), dim3(256), 0, stream, p, f); break;
        default: return GD_ENOKERNEL;
        }
#undef K_GEMM_NK
    } else {
        const uint64_t total = (uint64_t)p.M * p.N;
        uint64_t blocks = (total + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        GD_LAUNCH_VARIANT(variant, k_gemm_generic, dim3((uint32_t)blocks), dim3(256), stream, p, f);
    }
    GD_CHECK_LAUNCH();
    return GD_OK;
}

}  // namespace gd
