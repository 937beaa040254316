// C = A * B, bfloat16 operands, fp32 accumulation on the matrix cores, bfloat16
// result.  A is row-major M x K; B is stored N x K with K contiguous (b_is_nk) --
// both operands are then read as 16-byte runs along K -- or row-major K x N
// (handled by the generic kernel).  Tiles of A and B are staged through LDS; every
// global tile load and every store of C carries the fence on its final address.
// LDS is not fenced.
//
// Tiled kernels: one workgroup of 4 wavefronts (2 x 2) computes a 256 x 256 tile
// of C; each wavefront owns 128 x 128 of it (256 fp32 accumulators per lane, one
// wavefront per SIMD).  The finished tile is converted to bf16, transposed
// through LDS and stored as 16-byte runs.
//   k_gemm_ring  (shapes that are multiples of the tile, K % 128 == 0, operands
//                128-byte aligned: the measured path) v_mfma_f32_16x16x32_bf16; K
//                advances in slices of 32 through a ring of five 32 KiB LDS stages
//                filled by global_load_lds_dwordx4 (no staging registers, no LDS
//                store instructions); described in front of the kernel.
//   k_gemm_units (other multiples of the tile: K % 64 == 0, operands 16-byte
//                aligned) same MFMA shape and copies, a ring of five operand blocks
//                of K = 64 and one barrier per 64 k; as fast as k_gemm_ring when the
//                chip is not power limited, 1 % slower on N(0,1) data.
//   k_gemm_nk256 (ragged shapes) stages through registers so that out-of-range
//                rows and the K tail can be zero-filled.
//   k_gemm_generic  any shape, alignment and layout of B: one thread per entry.
#include "launchers.hpp"

namespace gd {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t gemm_f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// ---- generic kernel: any shape, any alignment, either layout of B -------------------
// One thread per entry of C, 2-byte accesses, fp32 accumulation in k order.  Under
// address checking the thread returns at its first refused access (counted once).
template <int V>
__global__ __launch_bounds__(256) void k_gemm_generic(gd_args_gemm p, FenceArgs fa)
{
    const Fence<V> F(fa);
    const uint64_t total = (uint64_t)p.M * p.N;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t e = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
        const uint64_t m = e / p.N, n = e % p.N;
        float acc = 0.0f;
        bool stopped = false;
        for (uint64_t k = 0; k < p.K; ++k) {
            const uint64_t aa = p.A + 2 * (m * p.K + k);
            const uint64_t ab = p.B + 2 * (p.b_is_nk ? n * p.K + k : k * p.N + n);
            if (!F.template inside<2>(aa) || !F.template inside<2>(ab)) { stopped = true; break; }
            const uint32_t ha = F.template ld<uint16_t>(aa);
            const uint32_t hb = F.template ld<uint16_t>(ab);
            acc += __uint_as_float(ha << 16) * __uint_as_float(hb << 16);
        }
        if (stopped || !F.template inside<2>(p.C + 2 * e)) { F.fault(); continue; }
        F.template st<uint16_t>(p.C + 2 * e, (uint16_t)gemm_f32_to_bf16(acc));
    }
}

// ---- tiled MFMA kernel ---------------------------------------------------------------
// Requirements (checked by the launcher): B stored N x K, K % 8 == 0, A and B
// 16-byte aligned.  EDGE = 0 additionally assumes M % 256 == 0, N % 256 == 0,
// K % 64 == 0, C 16-byte aligned: no predicates anywhere.
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int TM = 4, TN = 4;                       // MFMA tiles per wavefront
constexpr int STAGE_BYTES = (BM + BN) * BK * 2;     // 64 KiB
constexpr int A_BYTES = BM * BK * 2;                // 32 KiB
constexpr int LOADS = BM * (BK / 8) / 256;          // 16-byte granules per thread per operand: 8
constexpr int GROUP_M = 4;                          // tile rows walked together (L2 reuse)

template <int V, bool EDGE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void k_gemm_nk256(gd_args_gemm p, FenceArgs fa, uint32_t tiles_m, uint32_t tiles_n)
{
    const Fence<V> F(fa);
    __shared__ __attribute__((aligned(16))) uint8_t smem[2 * STAGE_BYTES];

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63, wave = tid >> 6;
    const uint32_t wm = wave >> 1, wn = wave & 1;

    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): give
    // every XCD a contiguous run of tiles, walked GROUP_M tile rows at a time.
    uint32_t lin = blockIdx.x;
    const uint32_t nblk = gridDim.x;
    if ((nblk & 7) == 0) lin = (lin & 7) * (nblk >> 3) + (lin >> 3);
    const uint32_t width = GROUP_M * tiles_n;
    const uint32_t first_m = (lin / width) * GROUP_M;
    const uint32_t gsize = (tiles_m - first_m < GROUP_M) ? tiles_m - first_m : GROUP_M;
    const uint32_t m0 = (first_m + (lin % width) % gsize) * BM;
    const uint32_t n0 = ((lin % width) / gsize) * BN;

    // global -> register -> LDS mapping: thread = (row t/8 + 32*i, granule t%8)
    const uint32_t lrow = tid >> 3, lg = tid & 7;
    const uint64_t a_ptr = p.A + 2 * ((uint64_t)(m0 + lrow) * p.K + lg * 8);
    const uint64_t b_ptr = p.B + 2 * ((uint64_t)(n0 + lrow) * p.K + lg * 8);
    const uint64_t row_step = 2 * 32 * (uint64_t)p.K;
    const uint32_t lds_w = lrow * 128 + ((lg ^ ((lrow >> 1) & 7)) << 4);

    // Address checking: thread (m, n) of C stops unless row m of A and column n of B
    // (a row of the N x K storage) are wholly inside the partition.  Rows that are not
    // are never read (they stay zero in LDS); their threads are counted at the store.
    const uint64_t run_bytes = 2 * (uint64_t)p.K;
    uint32_t a_live = 0, b_live = 0;             // bit i: this thread's i-th row of A / of B may be read
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
        a_live |= (uint32_t)F.inside_run(p.A + (uint64_t)(m0 + lrow + 32 * i) * run_bytes, run_bytes) << i;
        b_live |= (uint32_t)F.inside_run(p.B + (uint64_t)(n0 + lrow + 32 * i) * run_bytes, run_bytes) << i;
    }

    u32x4 ra[LOADS], rb[LOADS];
    auto gload = [&](uint32_t k0) {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            if (EDGE) {
                ra[i] = (u32x4){0, 0, 0, 0};
                rb[i] = (u32x4){0, 0, 0, 0};
                const bool kin = k0 + lg * 8 < p.K;
                if (kin && m0 + lrow + 32 * i < p.M && ((a_live >> i) & 1)) ra[i] = F.template ld<u32x4>(a_ptr + i * row_step + 2 * (uint64_t)k0);
                if (kin && n0 + lrow + 32 * i < p.N && ((b_live >> i) & 1)) rb[i] = F.template ld<u32x4>(b_ptr + i * row_step + 2 * (uint64_t)k0);
            } else {
                ra[i] = F.template ld<u32x4>(a_ptr + i * row_step + 2 * (uint64_t)k0);
                rb[i] = F.template ld<u32x4>(b_ptr + i * row_step + 2 * (uint64_t)k0);
            }
        }
    };
    auto lstore = [&](uint32_t stage) {
        uint8_t *sa = smem + stage * STAGE_BYTES + lds_w;
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            *(u32x4 *)(sa + i * 32 * 128) = ra[i];
            *(u32x4 *)(sa + A_BYTES + i * 32 * 128) = rb[i];
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // fragment addresses: lane = (row l%32, k half l/32); granule (2*kk + half) ^ ((row/2) & 7)
    const uint32_t frow = lane & 31, fhalf = lane >> 5;
    const uint32_t a_frag = (wm * 128 + frow) * 128;
    const uint32_t b_frag = A_BYTES + (wn * 128 + frow) * 128;
    uint32_t gsw[BK / 16];
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) gsw[kk] = ((2 * kk + fhalf) ^ ((frow >> 1) & 7)) << 4;

    const uint32_t ksteps = (p.K + BK - 1) / BK;
    gload(0);
    lstore(0);
    if (ksteps > 1) gload(BK);
    __syncthreads();

    for (uint32_t t = 0; t < ksteps; ++t) {
        const uint8_t *st = smem + (t & 1) * STAGE_BYTES;
        if (t + 1 < ksteps) lstore((t + 1) & 1);          // tile t+1: registers -> other stage
        if (t + 2 < ksteps) gload((t + 2) * BK);          // tile t+2: global -> registers
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 fa_[TM], fb_[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa_[i] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(st + a_frag + i * 32 * 128 + gsw[kk]));
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb_[j] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(st + b_frag + j * 32 * 128 + gsw[kk]));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa_[i], fb_[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // Epilogue.  acc[i][j][r] is C[row, col] of the wavefront's block with
    // row = 32*i + 8*(r/4) + 4*(lane/32) + r%4, col = 32*j + lane%32.  Each
    // wavefront parks its 128 x 128 bf16 block in its own 32 KiB of LDS (rows of
    // 256 bytes), then streams it out as 16-byte runs: 16 lanes cover one row.
    uint8_t *park = smem + wave * (128 * 256);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {                 // rows r and r + 1 of the same column: one packed conversion
                const f32x2 two = {acc[i][j][r], acc[i][j][r + 1]};
                const uint32_t w = __builtin_bit_cast(uint32_t, __builtin_convertvector(two, bf16x2));
                const uint32_t row = 32 * i + 8 * (r / 4) + 4 * fhalf + (r & 3);
                const uint32_t col = 32 * j + frow;
                *(uint16_t *)(park + row * 256 + col * 2) = (uint16_t)w;
                *(uint16_t *)(park + (row + 1) * 256 + col * 2) = (uint16_t)(w >> 16);
            }
    __syncthreads();
    const uint32_t orow = lane >> 4, og = lane & 15;
    const bool vec_ok = !EDGE || (((p.C & 15) == 0) && ((p.N & 7) == 0));
    // Address checking: which of this lane's eight columns of B are wholly inside.
    uint32_t col_live = 0xff;
    if (F.CHECKED) {
        col_live = 0;
        for (int e = 0; e < 8; ++e)
            col_live |= (uint32_t)F.inside_run(p.B + (uint64_t)(n0 + wn * 128 + og * 8 + e) * run_bytes, run_bytes) << e;
    }
    uint32_t stopped = 0;
#pragma unroll 4
    for (int it = 0; it < 32; ++it) {
        const uint32_t row = orow + 4 * it;
        const uint32_t m = m0 + wm * 128 + row, n = n0 + wn * 128 + og * 8;
        const u32x4 v = *(const u32x4 *)(park + row * 256 + og * 16);
        const uint64_t dst = p.C + 2 * ((uint64_t)m * p.N + n);
        if (!EDGE) {
            F.template st<u32x4, true>(dst, v);
        } else if (m < p.M && n < p.N) {
            const bool row_live = F.inside_run(p.A + (uint64_t)m * run_bytes, run_bytes);
            if (vec_ok && n + 8 <= p.N && row_live && col_live == 0xff && F.template inside<16>(dst)) {
                F.template st<u32x4, true>(dst, v);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (n + e < p.N) {
                        if (row_live && ((col_live >> e) & 1) && F.template inside<2>(dst + 2 * e))
                            F.template st<uint16_t>(dst + 2 * e, (uint16_t)(v[e >> 1] >> ((e & 1) * 16)));
                        else
                            ++stopped;
                    }
            }
        }
    }
    if (F.CHECKED && stopped) F.fault(stopped);
}


#define GD_LDS __attribute__((address_space(3)))

// ---- tiled MFMA kernel, five-stage ring of K=32 slices -----------------------------------------
// 256 x 256 tile, 2 x 2 wavefronts of 128 x 128 each.  K advances in
// slices of 32 through a ring of five 32 KiB LDS stages (A 256x32 + B 256x32),
// all 160 KiB of the compute unit.  LDS rows are 64 bytes; granule g of row r sits
// in slot g ^ ring_swizzle(r/4).
//
// A 64-byte row of a slice is half of a 128-byte cache line, and the L2 serves
// one request per channel and clock whether it asks for 64 or 128 bytes.  Slices
// are therefore requested in pairs (2j, 2j+1) whose rows together are whole lines:
// the two DMA instructions for the halves of the same rows are issued back to
// back, and the vector cache merges them into one 128-byte request (half the L2
// requests per byte).
//
// The global -> LDS path of a compute unit delivers little more than the 32 bytes
// per clock this tile shape consumes, and a wavefront that issues a DMA while the
// path is backed up stalls, MFMAs included.  The 16 DMAs of a pair of slices are
// therefore spread evenly over the two steps (32 MFMA pairs) in which both target
// stages are free: pair (t+3, t+4), t odd, goes out between the barrier of step
// t-1 and the barrier of step t+1, two DMAs every fourth MFMA pair.
// Requirements: M and N multiples of 256, K % 128 == 0, K <= 2^22, B stored N x K,
// A and B 128-byte aligned, C 16-byte aligned.
constexpr int RK = 32;                       // K per ring step
constexpr int RSTAGE = (BM + BN) * RK * 2;   // 32 KiB
constexpr int RA = BM * RK * 2;              // 16 KiB: offset of the B slice inside a stage

constexpr int RT = 8;                        // 16 x 16 MFMA tiles per wavefront, each way

// Slot permutation of the ring's LDS rows.  A fragment load (ds_read_b128) has lane l
// read row l%16, granule l/16.  The LDS serves a 128-bit read 16 lanes at a time, and
// not in lane order: lanes {0-3, 12-15, 20-23, 24-27} go together, then {4-7, 8-11,
// 16-19, 28-31}, then the same two sets plus 32 (measured: with the plain
// (r/4) & 3 swizzle SQ_LDS_BANK_CONFLICT counts 4 extra cycles per load, exactly
// what this grouping predicts, and none with 32 rows per granule column).  Rows 64
// bytes apart by a multiple of 4 rows share their banks, so within each set the four
// rows r, r+4, r+8, r+12 -- which come with granules (0,1,1,0) in the first set and
// (1,0,0,1) in the second -- must land in four different slots.  The permutation
// 0,2,3,1 of r/4 does that for all four sets.
__device__ __forceinline__ uint32_t ring_swizzle(uint32_t row_div4)
{
    return (0x78u >> (2 * (row_div4 & 3))) & 3;
}

// Workgroup barrier of the ring: wait until at most `vm` of this wavefront's DMA
// loads are still in flight (they complete in order, so everything older has
// landed in LDS) and all its LDS reads have returned, then meet the other
// wavefronts.  The argument is the s_waitcnt immediate in gfx9 encoding:
// vmcnt[3:0] in bits 3:0 and vmcnt[5:4] in bits 15:14, expcnt (untouched, 7) in
// bits 6:4, lgkmcnt = 0 in bits 11:8.  The empty asm statements keep the
// compiler from moving LDS accesses across the barrier.
#define GD_WAIT_VM7 0x0077      // vmcnt <= 7
#define GD_WAIT_VM10 0x007A     // vmcnt <= 10
#define GD_WAIT_VM_ANY 0xC07F   // vmcnt <= 63: no constraint
#define GD_RING_BARRIER(imm)                    \
    do {                                        \
        __builtin_amdgcn_s_waitcnt(imm);        \
        asm volatile("" ::: "memory");          \
        __builtin_amdgcn_s_barrier();           \
        asm volatile("" ::: "memory");          \
    } while (0)

// WHOLE (modulo rule and address checking): the launcher has found that the fence maps A, B and C each to one
// contiguous range (Fence::whole_run; under address checking: that all three lie inside the partition, so that no
// logical thread can be refused).  The kernel repeats that test, fences the first byte of A and of B once on the
// scalar unit and addresses their tiles as "fenced start + offset" with the native kernel's DMA form -- the per-array
// fence of the streaming kernels applied to a matrix.  Without it these two rules pay per DMA address: the modulo
// rule 25 vector instructions (+17 % at 8192^3), address checking a predicated, register-staged kernel (+60 %).
template <int V, bool WHOLE = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void k_gemm_ring(gd_args_gemm p, FenceArgs fa, uint32_t tiles_m, uint32_t tiles_n)
{
    const Fence<V> F(fa);
    using DmaFence = Fence<WHOLE ? (int)V_NONE : V>;        // WHOLE: the tile addresses are sums with a fenced start
    const DmaFence D(fa);
    uint64_t a_start = p.A, b_start = p.B;
    if constexpr (WHOLE) {
        if (!(F.whole_run(p.A, 2 * (uint64_t)p.M * p.K) && F.whole_run(p.B, 2 * (uint64_t)p.N * p.K) &&
              F.whole_run(p.C, 2 * (uint64_t)p.M * p.N)))
            return;                                             // never taken: the launcher tested the same
        a_start = F.scalar_fence(p.A);
        b_start = F.scalar_fence(p.B);
    }
    // Separate arrays, so that the compiler can tell a fragment load from one stage
    // apart from a DMA into another and does not wait for the DMA.
    __shared__ __attribute__((aligned(1024))) uint8_t ring0[RSTAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t ring1[RSTAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t ring2[RSTAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t ring3[RSTAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t ring4[RSTAGE];

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t wm = wave >> 1, wn = wave & 1;

    uint32_t lin = blockIdx.x;
    const uint32_t nblk = gridDim.x;
    if ((nblk & 7) == 0) lin = (lin & 7) * (nblk >> 3) + (lin >> 3);
    const uint32_t width = GROUP_M * tiles_n;
    const uint32_t first_m = (lin / width) * GROUP_M;
    const uint32_t gsize = (tiles_m - first_m < GROUP_M) ? tiles_m - first_m : GROUP_M;
    const uint32_t m0 = (first_m + (lin % width) % gsize) * BM;
    const uint32_t n0 = ((lin % width) / gsize) * BN;

    // One DMA instruction fills 1 KiB = 16 slice rows; lane l lands in row l/4, slot
    // l%4, and fetches granule (l%4) ^ ring_swizzle(row/4) = (l%4) ^ ring_swizzle(l/16).  Wavefront
    // w moves rows [64w, 64w+64) of A and of B.  DMA number d of a pair of slices:
    // d/2 = operand and 16-row chunk (0..3 A, 4..7 B), d%2 = slice of the pair, so the
    // two halves of the same cache lines are neighbours in issue order.
    const uint32_t drow = wave * 64 + (lane >> 2);
    const uint32_t dgran = (lane & 3) ^ ring_swizzle(lane >> 4);
    const uint32_t lane_off = 2 * (drow * p.K + dgran * 8);     // below 2^32: the launcher bounds K
    const uint64_t a_tile = a_start + 2 * (uint64_t)m0 * p.K;
    const uint64_t b_tile = b_start + 2 * (uint64_t)n0 * p.K;
    const uint64_t chunk_step = 2 * 16 * (uint64_t)p.K;      // 16 rows further down
    // The two DMAs of a cache line share one fenced address: A, B and the row pitch
    // 2*K are multiples of 128 bytes and k_pair of 64 elements, so the address of the
    // first half is a multiple of 128 plus the lane's granule (bits 4..5), and the
    // second half, 64 bytes further, lies in the same fenced line (see
    // Fence::dma16_unordered).
    typename DmaFence::SplitHandle pre[8];                 // one fenced address per DMA pair of the set
    auto pre_one = [&](uint32_t k_pair, int pr) {
        const uint64_t uni = (pr < 4 ? a_tile : b_tile) + (pr & 3) * chunk_step + 2 * (uint64_t)k_pair;
        pre[pr] = D.template fenced_split<16>(uni, lane_off);
    };
    auto dma_one = [&](uint8_t *stage_even, uint8_t *stage_odd, int d) {
        const int c = d >> 1;
        uint8_t *stage = (d & 1) ? stage_odd : stage_even;
        GD_LDS uint8_t *dst = (GD_LDS uint8_t *)stage + wave * 4096 + (c & 3) * 1024 + (c < 4 ? 0 : RA);
        if (d & 1) D.template dma16_unordered<2 * RK>(pre[c], (uint32_t)(uintptr_t)dst);
        else D.template dma16_unordered<0>(pre[c], (uint32_t)(uintptr_t)dst);
    };

    // 8 x 8 tiles of 16 x 16 per wavefront, v_mfma_f32_16x16x32_bf16: one instruction
    // takes the whole K = 32 of a slice.  Per flop this shape moves half as many
    // accumulator registers as the 32x32x16 one, and the chip, which is power limited
    // under this load, sustains a clearly higher clock on it.
    f32x4 acc[RT][RT];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < RT; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0f;

    // Fragment i of an operand: lane l holds row 16*i + l%16, granule l/16 (8 of the
    // 32 k) -- one ds_read_b128.  (16*i)/4 is a multiple of 4, so the swizzle term of
    // a lane does not depend on i and fragments sit at immediate offsets of 1 KiB.
    const uint32_t l16 = lane & 15, lg = lane >> 4;
    const uint32_t gsw = (lg ^ ring_swizzle(l16 >> 2)) << 4;
    const uint32_t a_frag = (wm * 128 + l16) * 64 + gsw;
    const uint32_t b_frag = RA + (wn * 128 + l16) * 64 + gsw;
    bf16x8 fra[RT], fbx[RT], fby[RT];                     // B fragments are double-buffered across steps
    auto load_a = [&](const uint8_t *stage, int i) {
        fra[i] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(stage + a_frag + i * 1024));
    };
    auto load_b = [&](const uint8_t *stage, int j, bf16x8 (&fb_)[RT]) {
        fb_[j] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(stage + b_frag + j * 1024));
    };
    // Slot sl (0..15) of a step: A fragment sl/2 against B fragments 4*(sl%2)..+3.
    auto mfma_quad = [&](int sl, const bf16x8 (&fb_)[RT]) {
        const int i = sl >> 1;
#pragma unroll
        for (int j = 4 * (sl & 1); j < 4 * (sl & 1) + 4; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb_[j], fra[i], acc[i][j], 0, 0, 0);
    };
    // DMA pair number pr (0..7) of a pair of slices: operand and 16-row chunk pr,
    // both halves (prologue only: the steps below send the two halves two slots apart).
    auto dma_pair = [&](uint32_t k_pair, uint8_t *stage_even, uint8_t *stage_odd, int pr) {
        pre_one(k_pair, pr);
        dma_one(stage_even, stage_odd, 2 * pr);
        dma_one(stage_even, stage_odd, 2 * pr + 1);
    };
    // One ring step of 16 slots, four MFMAs (64 clocks) each.  In: fra[0..3] and all
    // of fb_cur hold fragments of `cur`.  Out: fra[0..3] and fb_nxt hold fragments of
    // `nxt`.  A fragments 4..7 of `cur` are fetched in slots 0..3 (first needed in
    // slot 8).  Behind the barrier, slots 10..13 fetch the 12 fragments the next step
    // starts with, in the order it needs them; fra[0..3] are dead by then.  Every
    // even slot sends one DMA: slots 0..10 the two halves of DMA pairs p0, p0+1, p0+2
    // of the slice pair (ea, oa, ka), slots 12 and 14 those of DMA pair p3 of the slice
    // pair (eb, ob, kb); the fenced address of a pair is computed in the slot of its
    // first half, before that slot's MFMAs.  An odd step t sends DMA pairs 1..4 of
    // slices (t+3, t+4); an even step t sends pairs 5..7 of slices (t+2, t+3) and pair 0
    // of slices (t+4, t+5), whose second stage is the one this step has just finished
    // reading.
    auto step = [&](const uint8_t *cur, const uint8_t *nxt, bf16x8 (&fb_cur)[RT], bf16x8 (&fb_nxt)[RT], bool odd,
                    uint8_t *ea, uint8_t *oa, uint32_t ka, uint8_t *eb, uint8_t *ob, uint32_t kb) {
        const int p0 = odd ? 1 : 5, p3 = odd ? 4 : 0;
#pragma unroll
        for (int sl = 0; sl < 16; ++sl) {
            if (sl == 10) {
                // Odd step t: slice t+1 must have landed, i.e. everything but the 7 DMAs
                // sent since slot 12 of step t-1.  Even step: `nxt` landed a step ago; the
                // barrier only releases the stage of `cur` for refilling.
                if (odd) GD_RING_BARRIER(GD_WAIT_VM7);
                else GD_RING_BARRIER(GD_WAIT_VM_ANY);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (sl < 4) load_a(cur, 4 + sl);
            if (sl == 10) { load_b(nxt, 0, fb_nxt); load_a(nxt, 0); load_b(nxt, 1, fb_nxt); }
            if (sl == 11) { load_b(nxt, 2, fb_nxt); load_b(nxt, 3, fb_nxt); load_b(nxt, 4, fb_nxt); }
            if (sl == 12) { load_b(nxt, 5, fb_nxt); load_b(nxt, 6, fb_nxt); load_b(nxt, 7, fb_nxt); }
            if (sl == 13) { load_a(nxt, 1); load_a(nxt, 2); load_a(nxt, 3); }
            // one DMA every second slot: DMA number 2*pr + h of the slice pair, h = sl/2 % 2
            if ((sl & 1) == 0) {
                const int pr = sl < 12 ? p0 + sl / 4 : p3;
                const int d = 2 * pr + ((sl >> 1) & 1);
                if ((d & 1) == 0) pre_one(sl < 12 ? ka : kb, pr);
                mfma_quad(sl, fb_cur);
                dma_one(sl < 12 ? ea : eb, sl < 12 ? oa : ob, d);
            } else {
                mfma_quad(sl, fb_cur);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    const uint32_t ksteps = p.K / RK;                    // multiple of 4
    const uint32_t k_last = p.K - 2 * RK;
    auto clamp_k = [&](uint32_t k) { return k < k_last ? k : k_last; };   // past the end: refetch the last pair, unused
#pragma unroll
    for (int pr = 0; pr < 8; ++pr) {                     // slices 0 and 1
        dma_pair(0, ring0, ring1, pr);
    }
#pragma unroll
    for (int pr = 0; pr < 5; ++pr) {                     // slices 2 and 3, DMA pairs 0..4
        dma_pair(clamp_k(2 * RK), ring2, ring3, pr);
    }
    GD_RING_BARRIER(GD_WAIT_VM10);                       // slices 0 and 1 have landed
#pragma unroll
    for (int j = 0; j < RT; ++j) load_b(ring0, j, fbx);
#pragma unroll
    for (int i = 0; i < 4; ++i) load_a(ring0, i);
    // Slice s lives in stage s % 5 and the DMA pattern has period 2, so the code
    // repeats every 10 steps; K % 128 == 0 lets the loop end after any odd step.
    for (uint32_t t = 0; t < ksteps;) {
        step(ring0, ring1, fbx, fby, false, ring2, ring3, clamp_k((t + 2) * RK), ring4, ring0, clamp_k((t + 4) * RK));
        step(ring1, ring2, fby, fbx, true, ring4, ring0, clamp_k((t + 4) * RK), ring4, ring0, clamp_k((t + 4) * RK));
        t += 2;
        if (t < ksteps) {
            step(ring2, ring3, fbx, fby, false, ring4, ring0, clamp_k((t + 2) * RK), ring1, ring2, clamp_k((t + 4) * RK));
            step(ring3, ring4, fby, fbx, true, ring1, ring2, clamp_k((t + 4) * RK), ring1, ring2, clamp_k((t + 4) * RK));
            t += 2;
        }
        if (t < ksteps) {
            step(ring4, ring0, fbx, fby, false, ring1, ring2, clamp_k((t + 2) * RK), ring3, ring4, clamp_k((t + 4) * RK));
            step(ring0, ring1, fby, fbx, true, ring3, ring4, clamp_k((t + 4) * RK), ring3, ring4, clamp_k((t + 4) * RK));
            t += 2;
        }
        if (t < ksteps) {
            step(ring1, ring2, fbx, fby, false, ring3, ring4, clamp_k((t + 2) * RK), ring0, ring1, clamp_k((t + 4) * RK));
            step(ring2, ring3, fby, fbx, true, ring0, ring1, clamp_k((t + 4) * RK), ring0, ring1, clamp_k((t + 4) * RK));
            t += 2;
        }
        if (t < ksteps) {
            step(ring3, ring4, fbx, fby, false, ring0, ring1, clamp_k((t + 2) * RK), ring2, ring3, clamp_k((t + 4) * RK));
            step(ring4, ring0, fby, fbx, true, ring2, ring3, clamp_k((t + 4) * RK), ring2, ring3, clamp_k((t + 4) * RK));
            t += 2;
        }
    }
    // The compiler does not know of the ring's DMAs: wait for the last ones by hand
    // (vmcnt = 0, lgkmcnt = 0) before the stages are reused to park the result.
    __builtin_amdgcn_s_waitcnt(0x0070);
    __syncthreads();                                     // every DMA has landed, every fragment is read

    // Epilogue.  The MFMAs take the B fragment as their row operand, so acc[i][j][r]
    // is C[row, col] of the wavefront's block with row = 16*i + lane%16 and
    // col = 16*j + 4*(lane/16) + r: four consecutive columns, i.e. 8 contiguous bytes
    // of bf16.  Wavefront w parks its 128 x 128 bf16 block in ring stage w (rows of
    // 256 bytes = 32 units of 8 bytes; unit u of row q is kept at u ^ 2*(q%16), so
    // that the 16 rows written together spread over the banks and the two units of
    // a 16-byte granule stay neighbours), then streams it out as 16-byte runs, 16
    // lanes per row, with nontemporal stores: C is not read again, and written with plain
    // stores it takes cache space from the operand panels, which are (8192^3: +2 %).
    uint8_t *park = wave == 0 ? ring0 : wave == 1 ? ring1 : wave == 2 ? ring2 : ring3;
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < RT; ++j) {
            const f32x2 lo = {acc[i][j][0], acc[i][j][1]};
            const f32x2 hi = {acc[i][j][2], acc[i][j][3]};
            u32x2 w;
            w[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
            w[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
            const uint32_t row = 16 * i + l16;
            const uint32_t unit = (4 * j + lg) ^ (2 * l16);
            *(u32x2 *)(park + row * 256 + unit * 8) = w;
        }
    __syncthreads();
    const uint32_t orow = lane >> 4, og = lane & 15;
#pragma unroll 4
    for (int it = 0; it < 32; ++it) {
        const uint32_t row = orow + 4 * it;
        const uint32_t m = m0 + wm * 128 + row, n = n0 + wn * 128 + og * 8;
        const u32x4 v = *(const u32x4 *)(park + row * 256 + ((og ^ (row & 15)) << 4));
        F.template st<u32x4, true>(p.C + 2 * ((uint64_t)m * p.N + n), v);
    }
}

// ---- tiled MFMA kernel, ring of five operand blocks of K = 64 -----------------------------------
// Same tile, wavefront layout, MFMA shape and epilogue as k_gemm_ring.  The ring's
// unit is one operand block: 256 rows x 64 k (LDS rows of 128 bytes = whole cache
// lines, 32 KiB), A and B blocks alternating: unit n is A_{n/2} for even n, B_{n/2}
// for odd n, and lives in LDS slot n % 5.  One step takes K = 64 (two MFMA
// substeps, 128 MFMAs per wavefront) and one workgroup barrier, which does both
// jobs: it publishes the two units of the next step and it releases the two units
// just read, into which the DMAs for units 2j+5 and 2j+6 then go, one every second
// slot until the next barrier.  A DMA instruction moves 8 rows x 128 bytes.
// Granule g of row r sits in slot g ^ 2*h(r/2 % 8), h = 0,1,0,1,2,3,2,3: within each
// of the lane sets a 128-bit LDS read is served in (see ring_swizzle) the 8 rows
// of equal parity then use 8 different slots.
// Requirements: M and N multiples of 256, K % 64 == 0, K <= 2^22, B stored N x K,
// A, B and C 16-byte aligned.
constexpr int UK = 64;                       // K per step
constexpr int UBYTES = BM * UK * 2;          // 32 KiB per unit
constexpr int UBAR = 26;                     // slot (of 32) in front of which the barrier sits

__device__ __forceinline__ uint32_t unit_swizzle(uint32_t row)
{
    const uint32_t x = (row >> 1) & 7;
    return 2 * ((x & 1) | ((x >> 1) & 2));
}

// WHOLE: as in k_gemm_ring.
template <int V, bool WHOLE = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void k_gemm_units(gd_args_gemm p, FenceArgs fa, uint32_t tiles_m, uint32_t tiles_n)
{
    const Fence<V> F(fa);
    using DmaFence = Fence<WHOLE ? (int)V_NONE : V>;
    const DmaFence D(fa);
    uint64_t a_start = p.A, b_start = p.B;
    if constexpr (WHOLE) {
        if (!(F.whole_run(p.A, 2 * (uint64_t)p.M * p.K) && F.whole_run(p.B, 2 * (uint64_t)p.N * p.K) &&
              F.whole_run(p.C, 2 * (uint64_t)p.M * p.N)))
            return;                                             // never taken: the launcher tested the same
        a_start = F.scalar_fence(p.A);
        b_start = F.scalar_fence(p.B);
    }
    __shared__ __attribute__((aligned(1024))) uint8_t u0[UBYTES];
    __shared__ __attribute__((aligned(1024))) uint8_t u1[UBYTES];
    __shared__ __attribute__((aligned(1024))) uint8_t u2[UBYTES];
    __shared__ __attribute__((aligned(1024))) uint8_t u3[UBYTES];
    __shared__ __attribute__((aligned(1024))) uint8_t u4[UBYTES];

    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t wm = wave >> 1, wn = wave & 1;

    uint32_t lin = blockIdx.x;
    const uint32_t nblk = gridDim.x;
    if ((nblk & 7) == 0) lin = (lin & 7) * (nblk >> 3) + (lin >> 3);
    const uint32_t width = GROUP_M * tiles_n;
    const uint32_t first_m = (lin / width) * GROUP_M;
    const uint32_t gsize = (tiles_m - first_m < GROUP_M) ? tiles_m - first_m : GROUP_M;
    const uint32_t m0 = (first_m + (lin % width) % gsize) * BM;
    const uint32_t n0 = ((lin % width) / gsize) * BN;

    // DMA c (0..7) of a unit: wavefront w moves rows 64w + 8c + l/8; lane l lands in
    // slot l%8 of its row and fetches granule (l%8) ^ unit_swizzle(row).  (row/2) % 8 =
    // (4c + l/16) % 8, so there is one lane offset for even c and one for odd c.
    const uint32_t drow = wave * 64 + (lane >> 3);
    uint32_t lane_off[2];
#pragma unroll
    for (int par = 0; par < 2; ++par) {
        const uint32_t gran = (lane & 7) ^ unit_swizzle(8 * par + (lane >> 3));
        lane_off[par] = 2 * (drow * p.K + gran * 8);           // below 2^32: the launcher bounds K
    }
    const uint64_t a_tile = a_start + 2 * (uint64_t)m0 * p.K;
    const uint64_t b_tile = b_start + 2 * (uint64_t)n0 * p.K;
    const uint64_t chunk_step = 2 * 8 * (uint64_t)p.K;           // 8 rows further down
    typename DmaFence::SplitHandle pre;
    auto dma = [&](bool is_b, uint32_t k0, uint8_t *unit, int c) {
        const uint64_t uni = (is_b ? b_tile : a_tile) + c * chunk_step + 2 * (uint64_t)k0;
        pre = D.template fenced_split<16>(uni, lane_off[c & 1]);
        GD_LDS uint8_t *dst = (GD_LDS uint8_t *)unit + wave * 8192 + c * 1024;
        D.template dma16_unordered<0>(pre, (uint32_t)(uintptr_t)dst);
    };

    f32x4 acc[RT][RT];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < RT; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0f;

    // Fragment i of an operand, substep kk: lane l holds row 16*i + l%16, granule
    // 4*kk + l/16.  16*i is a multiple of 16, so the swizzle term of a lane does not
    // depend on i and fragments sit at immediate offsets of 2 KiB.
    const uint32_t l16 = lane & 15, lg = lane >> 4;
    uint32_t a_frag[2], b_frag[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        const uint32_t slot = ((4 * kk) | lg) ^ unit_swizzle(l16);
        a_frag[kk] = (wm * 128 + l16) * 128 + slot * 16;
        b_frag[kk] = (wn * 128 + l16) * 128 + slot * 16;
    }
    bf16x8 fra[RT], fbx[RT], fby[RT];        // A fragments; B fragments of substep 0 and of substep 1
    auto load_a = [&](const uint8_t *unit, int kk, int i) {
        fra[i] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(unit + a_frag[kk] + i * 2048));
    };
    auto load_b = [&](const uint8_t *unit, int kk, int j, bf16x8 (&fb_)[RT]) {
        fb_[j] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(unit + b_frag[kk] + j * 2048));
    };
    auto mfma_quad = [&](int sl, const bf16x8 (&fb_)[RT]) {
        const int i = sl >> 1;
#pragma unroll
        for (int j = 4 * (sl & 1); j < 4 * (sl & 1) + 4; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb_[j], fra[i], acc[i][j], 0, 0, 0);
    };
    // One step of 32 slots, four MFMAs (64 clocks) each: slots 0..15 substep 0 (fbx),
    // slots 16..31 substep 1 (fby).  In: fra[0..3] and fbx hold substep-0 fragments of
    // (ac, bc).  Out: the same for (an, bn).
    // Fragment loads: A 4..7 of substep 0 in slots 0..3; B of substep 1 in slots 4..11,
    // A 0..3 of substep 1 in slots 8..11 (their registers are free from slot 8), A 4..7
    // of substep 1 in slots 16..19; behind the barrier, slots 26..29, the 12 fragments
    // the next step starts with.
    // DMAs, one every second slot: slots 0..8 finish unit B_{j+1} (DMAs 3..7; its first
    // three went out behind the previous barrier), slots 10..24 send A_{j+2}, slots
    // 26..30 start B_{j+2} in the unit A_j has just left.
    auto step = [&](const uint8_t *ac, const uint8_t *bc, const uint8_t *an, uint8_t *bn, uint8_t *a2,
                    uint8_t *ac_w, uint32_t k1, uint32_t k2) {
#pragma unroll
        for (int sl = 0; sl < 32; ++sl) {
            if (sl == UBAR) {
                // Units A_{j+1}, B_{j+1} must have landed: everything but the 8 DMAs of
                // A_{j+2}.  All fragment loads of this step have been issued by slot 19.
                GD_RING_BARRIER(0x0078);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (sl < 4) load_a(ac, 0, 4 + sl);
            if (sl >= 4 && sl < 12) load_b(bc, 1, sl - 4, fby);
            if (sl >= 8 && sl < 12) load_a(ac, 1, sl - 8);
            if (sl >= 16 && sl < 20) load_a(ac, 1, 4 + sl - 16);
            if (sl == UBAR) { load_b(bn, 0, 0, fbx); load_a(an, 0, 0); load_b(bn, 0, 1, fbx); }
            if (sl == UBAR + 1) { load_b(bn, 0, 2, fbx); load_b(bn, 0, 3, fbx); load_b(bn, 0, 4, fbx); }
            if (sl == UBAR + 2) { load_b(bn, 0, 5, fbx); load_b(bn, 0, 6, fbx); load_b(bn, 0, 7, fbx); }
            if (sl == UBAR + 3) { load_a(an, 0, 1); load_a(an, 0, 2); load_a(an, 0, 3); }
            if (sl < 16) mfma_quad(sl, fbx);
            else mfma_quad(sl - 16, fby);
            if ((sl & 1) == 0) {
                constexpr int NB = (32 - UBAR) / 2;            // DMAs of B_{j+2} sent behind the barrier
                if (sl >= UBAR) dma(true, k2, ac_w, (sl - UBAR) / 2);
                else if (sl / 2 < 8 - NB) dma(true, k1, bn, NB + sl / 2);
                else if (sl / 2 < 16 - NB) dma(false, k2, a2, sl / 2 - (8 - NB));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    const uint32_t nsteps = p.K / UK;
    const uint32_t k_last = p.K - UK;
    auto clamp_k = [&](uint32_t k) { return k < k_last ? k : k_last; };   // past the end: refetch the last block, unused
#pragma unroll
    for (int c = 0; c < 8; ++c) dma(false, 0, u0, c);                    // A_0
#pragma unroll
    for (int c = 0; c < 8; ++c) dma(true, 0, u1, c);                     // B_0
#pragma unroll
    for (int c = 0; c < 8; ++c) dma(false, clamp_k(UK), u2, c);          // A_1
#pragma unroll
    for (int c = 0; c < (32 - UBAR) / 2; ++c) dma(true, clamp_k(UK), u3, c);   // B_1, its first DMAs
    GD_RING_BARRIER(0x0078 + (32 - UBAR) / 2);                           // vmcnt <= 8 + those: A_0 and B_0 have landed
#pragma unroll
    for (int j = 0; j < RT; ++j) load_b(u1, 0, j, fbx);
#pragma unroll
    for (int i = 0; i < 4; ++i) load_a(u0, 0, i);
    // Unit n lives in u[n % 5]: step j reads u[2j % 5] and u[(2j+1) % 5], the next step's
    // units are the two after them, A_{j+2} goes into the fifth.  Period: 5 steps.
    for (uint32_t j = 0; j < nsteps;) {
        step(u0, u1, u2, u3, u4, u0, clamp_k((j + 1) * UK), clamp_k((j + 2) * UK));
        ++j;
        if (j < nsteps) { step(u2, u3, u4, u0, u1, u2, clamp_k((j + 1) * UK), clamp_k((j + 2) * UK)); ++j; }
        if (j < nsteps) { step(u4, u0, u1, u2, u3, u4, clamp_k((j + 1) * UK), clamp_k((j + 2) * UK)); ++j; }
        if (j < nsteps) { step(u1, u2, u3, u4, u0, u1, clamp_k((j + 1) * UK), clamp_k((j + 2) * UK)); ++j; }
        if (j < nsteps) { step(u3, u4, u0, u1, u2, u3, clamp_k((j + 1) * UK), clamp_k((j + 2) * UK)); ++j; }
    }
    // The compiler does not know of the ring's DMAs: wait for the last ones by hand
    // (vmcnt = 0, lgkmcnt = 0) before the units are reused to park the result.
    __builtin_amdgcn_s_waitcnt(0x0070);
    __syncthreads();

    // Epilogue: as in k_gemm_ring.
    uint8_t *park = wave == 0 ? u0 : wave == 1 ? u1 : wave == 2 ? u2 : u3;
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < RT; ++j) {
            const f32x2 lo = {acc[i][j][0], acc[i][j][1]};
            const f32x2 hi = {acc[i][j][2], acc[i][j][3]};
            u32x2 w;
            w[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
            w[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
            const uint32_t row = 16 * i + l16;
            const uint32_t unit = (4 * j + lg) ^ (2 * l16);
            *(u32x2 *)(park + row * 256 + unit * 8) = w;
        }
    __syncthreads();
    const uint32_t orow = lane >> 4, og = lane & 15;
#pragma unroll 4
    for (int it = 0; it < 32; ++it) {
        const uint32_t row = orow + 4 * it;
        const uint32_t m = m0 + wm * 128 + row, n = n0 + wn * 128 + og * 8;
        const u32x4 v = *(const u32x4 *)(park + row * 256 + ((og ^ (row & 15)) << 4));
        F.template st<u32x4, true>(p.C + 2 * ((uint64_t)m * p.N + n), v);
    }
}

// ---- measurement aid: what the matrix pipe sustains with no data movement at all ---------------
// The wavefront layout and MFMA order of the ring kernel (8 x 8 tiles of 16x16x32, 256
// accumulators per lane, one wavefront per SIMD) with both operands held in registers:
// no LDS, no global traffic inside the loop.  Under the chip's power limit the rate of
// this loop on N(0,1) operands is the ceiling any GEMM on such data can approach.
// `operands`: 16 fragments x 256 threads x 16 bytes of bf16 (64 KiB), caller-owned.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void k_mfma_probe(const u32x4 *operands, float *out, uint32_t iters)
{
    bf16x8 fa[RT], fb[RT];
#pragma unroll
    for (int i = 0; i < RT; ++i) {
        fa[i] = __builtin_bit_cast(bf16x8, operands[threadIdx.x + 256 * i]);
        fb[i] = __builtin_bit_cast(bf16x8, operands[threadIdx.x + 256 * (RT + i)]);
    }
    f32x4 acc[RT][RT];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < RT; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0f;
    for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int e = 0; e < RT * RT; ++e)
            acc[e / RT][e % RT] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[e % RT], fa[e / RT], acc[e / RT][e % RT], 0, 0, 0);
        const bf16x8 t = fa[0];                 // rotate, so that successive passes multiply other data
#pragma unroll
        for (int i = 0; i + 1 < RT; ++i) fa[i] = fa[i + 1];
        fa[RT - 1] = t;
    }
    // every accumulator is "used" (so that no MFMA chain is dead code) without arithmetic on all 256
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < RT; ++j) asm volatile("" : : "v"(acc[i][j]));
    out[(uint64_t)blockIdx.x * 256 + threadIdx.x] = acc[0][0][0] + acc[RT - 1][RT - 1][3];
}

int launch_mfma_probe(uint64_t operands, uint64_t out, uint32_t blocks, uint32_t iters, hipStream_t stream)
{
    if (!operands || !out || (operands & 15) || (out & 3) || blocks == 0 || blocks > 65536) return GD_EINVAL;
    hipLaunchKernelGGL(k_mfma_probe, dim3(blocks), dim3(256), 0, stream, (const u32x4 *)(uintptr_t)operands,
                       (float *)(uintptr_t)out, iters);
    GD_CHECK_LAUNCH();
    return GD_OK;
}

// ---- launcher ---------------------------------------------------------------------------

int launch_gemm_bf16(const void *args, const FenceArgs &f, int variant, const Shape &shape,
                     hipStream_t stream)
{
    const gd_args_gemm &p = *(const gd_args_gemm *)args;
    if (shape.grid || shape.block) return GD_EINVAL;
    if (p.M == 0 || p.N == 0) return GD_OK;
    const bool tiled = p.b_is_nk && p.K > 0 && (p.K % 8) == 0 && ((p.A | p.B) & 15) == 0;
    int rc;
    if (tiled) {
        const uint32_t tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
        const uint64_t tiles = (uint64_t)tiles_m * tiles_n;
        if (tiles > 0x7fffffffull) return GD_ESHAPE;
        // the ring kernels keep per-lane byte offsets of up to 256 rows in 32 bits
        const bool edge = (p.M % BM) || (p.N % BN) || (p.K % BK) || (p.C & 15) || p.K > (1u << 22);
        const bool ring = p.K % 128 == 0 && ((p.A | p.B) & 127) == 0;
        const dim3 grid((uint32_t)tiles), block(256);
        rc = with_variant(variant, [&](auto v) {
            constexpr int V = decltype(v)::value;
            // address checking needs predicated loads, and the hardware-checked rule buffer
            // instructions: the register-staged kernel has both
            if constexpr (V == V_MOD || V == V_CHECK) {
                // every operand mapped to one contiguous range (all inside, for address checking): fence each once
                if (!edge && whole_run_host(f, V, p.A, 2 * (uint64_t)p.M * p.K) && whole_run_host(f, V, p.B, 2 * (uint64_t)p.N * p.K) &&
                    whole_run_host(f, V, p.C, 2 * (uint64_t)p.M * p.N)) {
                    if (ring) hipLaunchKernelGGL((k_gemm_ring<V, true>), grid, block, 0, stream, p, f, tiles_m, tiles_n);
                    else hipLaunchKernelGGL((k_gemm_units<V, true>), grid, block, 0, stream, p, f, tiles_m, tiles_n);
                    return;
                }
            }
            if constexpr (V == V_BUF) {
                // buffer offsets add up by definition: the ring's copies become buffer loads to the LDS, range-checked per lane
                if (!edge) {
                    if (ring) hipLaunchKernelGGL((k_gemm_ring<V, false>), grid, block, 0, stream, p, f, tiles_m, tiles_n);
                    else hipLaunchKernelGGL((k_gemm_units<V, false>), grid, block, 0, stream, p, f, tiles_m, tiles_n);
                    return;
                }
            }
            if (V == V_CHECK || V == V_BUF || edge) {
                hipLaunchKernelGGL((k_gemm_nk256<V, true>), grid, block, 0, stream, p, f, tiles_m, tiles_n);
            } else if constexpr (V != V_CHECK && V != V_BUF) {
                if (ring) hipLaunchKernelGGL((k_gemm_ring<V>), grid, block, 0, stream, p, f, tiles_m, tiles_n);
                else hipLaunchKernelGGL((k_gemm_units<V>), grid, block, 0, stream, p, f, tiles_m, tiles_n);
            }
        });
    } else {
        const uint64_t total = (uint64_t)p.M * p.N;
        uint64_t blocks = (total + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        rc = with_variant(variant, [&](auto v) {
            hipLaunchKernelGGL((k_gemm_generic<decltype(v)::value>), dim3((uint32_t)blocks), dim3(256), 0, stream, p, f);
        });
    }
    if (rc != GD_OK) return rc;
    GD_CHECK_LAUNCH();
    return GD_OK;
}

}  // namespace gd
