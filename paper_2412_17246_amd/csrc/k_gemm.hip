// Projections of a decoder layer: C[M,N] = A[M,K] * W[N,K]^T with bf16 inputs, fp32 accumulation on
// the matrix cores (v_mfma_f32_32x32x16_bf16), and three epilogues: plain, + residual, SwiGLU.
//
// Both operands are K-contiguous, so a lane's MFMA operand (8 consecutive k of one row / column)
// is one 16-byte LDS read.  Three kernels share the work: gemm_big_kernel (prefill-sized problems: 256x256
// tiles, operands global -> LDS by DMA into a five-slot ring), gemm_skinny_kernel (up to 256 rows: the
// weights are streamed once, split over K) and gemm_kernel below (everything else: K tails, odd widths,
// no workspace), which stages tiles global -> registers -> LDS, double buffered, one barrier per 64-wide
// K step, LDS rows padded by 16 bytes so that the operand reads of 16 consecutive rows fall in distinct banks.
#include <type_traits>

#include "common.h"

namespace bz {

// silu(z) = z / (1 + exp(-z)) with the hardware's exponential and reciprocal (about 1 ulp each; every
// use rounds the product to bf16 afterwards).  An IEEE division costs ten instructions per element in the
// epilogue of the gate/up projection, which has 128 of them per lane and tile.  One definition for every
// kernel that applies SwiGLU, so that they agree bit for bit.
__device__ __forceinline__ float silu_fast(float z) { return z * __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }

#ifndef BZ_FP32_DEBUG

constexpr int kBK = 64;            // K step per LDS stage
constexpr int kLdsRow = kBK + 8;   // padded row length in elements (144 bytes)

template <int BM, int BN>
constexpr int gemm_lds_bytes() { return 2 * (BM + BN) * kLdsRow * (int)sizeof(bf16); }

// Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of logical tile
// ids so tiles that share operand rows meet in one L2.
__device__ __forceinline__ int xcd_remap(int bid, int nb) {
    const int xcd = bid & 7, local = bid >> 3;
    const int base = nb >> 3, rem = nb & 7;
    return xcd * base + (xcd < rem ? xcd : rem) + local;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int MODE>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void gemm_kernel(const bf16* __restrict__ A,
                                                                      const bf16* __restrict__ W,
                                                                      const bf16* R, bf16* C, int M, int N,
                                                                      int K, int tiles_m, int tiles_n) {
    constexpr int THREADS = WAVES_M * WAVES_N * 64;
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    constexpr int MI = WTM / 32, NJ = WTN / 32;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of the MFMA block");
    static_assert(MODE != 2 || NJ % 2 == 0, "SwiGLU needs gate and up blocks in the same wave");
    constexpr int ROWS_PER_PASS = THREADS / 8;      // 8 vectors of 8 elements per 64-wide row
    constexpr int PA = BM / ROWS_PER_PASS, PB = BN / ROWS_PER_PASS;
    static_assert(BM % ROWS_PER_PASS == 0 && BN % ROWS_PER_PASS == 0, "tile rows vs loader passes");
    constexpr int OUT_BN = (MODE == 2) ? BN / 2 : BN;   // output columns per tile

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16* As = reinterpret_cast<bf16*>(smem_raw);                 // [2][BM][kLdsRow]
    bf16* Bs = As + 2 * BM * kLdsRow;                             // [2][BN][kLdsRow]

    // ---- tile coordinates (grouped along M for L2 reuse of the weight tile) ----
    const int pid = xcd_remap(blockIdx.x, tiles_m * tiles_n);
    constexpr int GROUP = 8;
    const int width = GROUP * tiles_n;
    const int group_id = pid / width;
    const int first_m = group_id * GROUP;
    const int gsize = (tiles_m - first_m < GROUP) ? (tiles_m - first_m) : GROUP;
    const int tile_m = first_m + (pid % width) % gsize;
    const int tile_n = (pid % width) / gsize;
    const int m0 = tile_m * BM;
    const int n0 = tile_n * OUT_BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int lrow = lane & 31, lk = lane >> 5;

    // ---- loader mapping ----
    const int vcol = tid & 7;             // which 8-element vector of the 64-wide row
    const int vrow = tid >> 3;            // row within a pass
    const bf16* a_ptr[PA];
    const bf16* b_ptr[PB];
#pragma unroll
    for (int p = 0; p < PA; ++p) {
        int r = m0 + vrow + p * ROWS_PER_PASS;
        if (r > M - 1) r = M - 1;
        a_ptr[p] = A + (size_t)r * K + vcol * 8;
    }
#pragma unroll
    for (int p = 0; p < PB; ++p) {
        const int lr = vrow + p * ROWS_PER_PASS;      // row in the LDS B tile
        int r;
        if (MODE == 2) {
            const bool up = lr >= BN / 2;
            int f = n0 + (up ? lr - BN / 2 : lr);
            if (f > N - 1) f = N - 1;
            r = up ? N + f : f;
        } else {
            r = n0 + lr;
            if (r > N - 1) r = N - 1;
        }
        b_ptr[p] = W + (size_t)r * K + vcol * 8;
    }

    uint4 ra[PA], rb[PB];
    auto load_tile = [&](int k0) {
        const bool kin = (k0 + vcol * 8) < K;
#pragma unroll
        for (int p = 0; p < PA; ++p)
            ra[p] = kin ? *reinterpret_cast<const uint4*>(a_ptr[p] + k0) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int p = 0; p < PB; ++p)
            rb[p] = kin ? *reinterpret_cast<const uint4*>(b_ptr[p] + k0) : make_uint4(0, 0, 0, 0);
    };
    auto store_tile = [&](int buf) {
        bf16* as = As + buf * BM * kLdsRow;
        bf16* bs = Bs + buf * BN * kLdsRow;
#pragma unroll
        for (int p = 0; p < PA; ++p)
            *reinterpret_cast<uint4*>(as + (vrow + p * ROWS_PER_PASS) * kLdsRow + vcol * 8) = ra[p];
#pragma unroll
        for (int p = 0; p < PB; ++p)
            *reinterpret_cast<uint4*>(bs + (vrow + p * ROWS_PER_PASS) * kLdsRow + vcol * 8) = rb[p];
    };

    f32x16 acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // LDS row of the wave's j-th column block
    int brow[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        if (MODE == 2) {
            constexpr int HJ = NJ / 2 > 0 ? NJ / 2 : 1;
            const bool up = j >= HJ;
            const int jj = up ? j - HJ : j;
            brow[j] = (up ? BN / 2 : 0) + (wn * HJ + jj) * 32 + lrow;
        } else {
            brow[j] = (wn * NJ + j) * 32 + lrow;
        }
    }

    const int nk = (K + kBK - 1) / kBK;
    load_tile(0);
    store_tile(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) load_tile((kt + 1) * kBK);
        const bf16* as = As + cur * BM * kLdsRow;
        const bf16* bs = Bs + cur * BN * kLdsRow;
#pragma unroll
        for (int ks = 0; ks < kBK / 16; ++ks) {
            bf16x8 af[MI], bfr[NJ];
#pragma unroll
            for (int i = 0; i < MI; ++i)
                af[i] = *reinterpret_cast<const bf16x8*>(as + (wm * WTM + i * 32 + lrow) * kLdsRow + ks * 16 + lk * 8);
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                bfr[j] = *reinterpret_cast<const bf16x8*>(bs + brow[j] * kLdsRow + ks * 16 + lk * 8);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) store_tile(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane holds column (lane%32) and rows 8*(r/4) + 4*(lane/32) + r%4 of each block
    if (MODE == 2) {
        constexpr int HJ = NJ / 2 > 0 ? NJ / 2 : 1;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < HJ; ++j) {
                const int col = n0 + (wn * HJ + j) * 32 + lrow;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = m0 + wm * WTM + i * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
                    if (row < M && col < N) {
                        const float g = acc[i][j][r], u = acc[i][j + HJ][r];
                        const float sg = silu_fast(g);
                        C[(size_t)row * N + col] = (bf16)(sg * u);
                    }
                }
            }
    } else {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const int col = n0 + (wn * NJ + j) * 32 + lrow;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = m0 + wm * WTM + i * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
                    if (row < M && col < N) {
                        float v = acc[i][j][r];
                        if (MODE == 1) v += (float)R[(size_t)row * N + col];
                        C[(size_t)row * N + col] = (bf16)v;
                    }
                }
            }
    }
}

// ---------------------------------------------------------------------------------------------
// Large-tile kernel for prefill-sized problems (K a multiple of 64, N a multiple of 4):
// 256x256x64 workgroup tile, 4 waves, 128x128 per wave (256 accumulator registers).  Operands reach
// LDS by direct global->LDS loads (16 bytes per lane, no register staging).  A wave's load
// instruction writes 1 KiB of LDS in lane order, i.e. 8 rows of 128 bytes; bank conflicts are
// avoided by permuting WHICH 16-byte piece of its row each lane fetches (an XOR swizzle applied on
// the global side) and reading operands with the same permutation.  The weight tile feeds the
// MFMA's row operand and the activation tile its column operand, so a lane ends up with runs of
// consecutive output features of one token (8 with the row order described at big_row_feature:
// 16-byte stores), and gate/up of the same feature in the same lane for the SwiGLU epilogue.
//
// LDS is a ring of five 32 KiB slots, each holding one operand's 256 rows of one k-tile: the tile
// being multiplied, the next one, and the activation half of the one after.  What decides the
// schedule is the cost of ISSUING a load: a 1 KiB load holds its wave's instruction stream for
// about 64 cycles when the four waves issue together (the address unit is shared), and a wave that
// cannot issue cannot feed the matrix pipe either.  So loads go out one every four MFMAs, spread
// over the whole tile, into the two slots the previous tile released, and the wait before a
// tile's barrier leaves the newest 32 KiB in flight.
// ---------------------------------------------------------------------------------------------
constexpr int kBigSlot = 256 * kBK * (int)sizeof(bf16);      // 32768: one operand's 256 rows of one k-tile
constexpr int kBigSlots = 5;

__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// Waves along the output-feature dimension: 2, i.e. four waves of 128x128 each, one per SIMD.  (Four - eight
// waves of 128x64, two per SIMD - was measured slower: its LDS operand reads fill the LDS port.)
constexpr int kBigWN = 2;

// logical tile id -> tile coordinates: groups of 4 tile rows, walked column by column, so that the
// tiles running together on an XCD share operand rows in its L2
// Which feature sits where.  A 32x32x16 MFMA leaves lane half h of the output with rows 8g + 4h + 0..3 of
// the row operand (register group g = registers 4g..4g+3).  The weight rows of a 32-feature block are
// therefore laid into LDS in a permuted order - operand row 8g + 4h + e holds feature
// 16*(g/2) + 8h + 4*(g%2) + e - so that a lane's registers 8p..8p+7 are the 8 consecutive features
// 16p + 8h + 0..7 of one token: 16-byte output stores, 32 contiguous bytes per token and instruction.  (In
// operand-row order a lane would own 4 consecutive features; the L2 then takes the output as twice as many
// partial-line writes, which is what bounds the epilogue.)  The permutation costs nothing: it only changes
// which global row a loader lane fetches.
__device__ __forceinline__ int big_row_feature(int rho) {            // operand row inside a block -> feature inside it
    const int g = rho >> 3, h = (rho >> 2) & 1, e = rho & 3;
    return 16 * (g >> 1) + 8 * h + 4 * (g & 1) + e;
}
__device__ __forceinline__ int big_group_feature(int g, int h) {     // first feature of register group g, lane half h
    return 16 * (g >> 1) + 8 * h + 4 * (g & 1);
}

struct BigTile { int m0, n0; };
template <int MODE>
__device__ __forceinline__ BigTile big_tile_of(int pid, int tiles_m, int tiles_n) {
    constexpr int OUT_BN = (MODE == 2) ? 128 : 256;
    constexpr int GROUP = 4;
    const int width = GROUP * tiles_n;
    const int group_id = pid / width;
    const int first_m = group_id * GROUP;
    const int gsize = (tiles_m - first_m < GROUP) ? (tiles_m - first_m) : GROUP;
    const int tile_m = first_m + (pid % width) % gsize;
    const int tile_n = (pid % width) / gsize;
    return BigTile{tile_m * 256, tile_n * OUT_BN};
}

// Output of one 32-token block of a wave: lane holds token m and, of each 32-feature block j,
// features fbase[j] + 8*g + 4*lk + 0..3 (accumulator registers 4g..4g+3).
// `get(j, x)` returns accumulator register x of block j (a callable, so the caller's registers are read in place).
template <int MODE, int NJ, class Get>
__device__ __forceinline__ void big_store_block(Get get, int m, int n0, const int (&fbase)[NJ], int lk,
                                                const bf16* R, bf16* C, int M, int N) {
    if (m >= M) return;
    bf16* crow = C + (size_t)m * N;
    if ((N & 7) == 0 && MODE != 1) {                 // rows 16-byte aligned: 8 features (registers 8p..8p+7) per store
        constexpr int NJE = (MODE == 2) ? NJ / 2 : NJ;
#pragma unroll
        for (int j = 0; j < NJE; ++j)
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const int n = n0 + fbase[j] + 16 * p + 8 * lk;
                if (n < N) {
                    bf16x8 o;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float v = get(j, 8 * p + e);
                        if (MODE == 2) o[e] = (bf16)(silu_fast(v) * get(j + NJ / 2, 8 * p + e));
                        else o[e] = (bf16)v;
                    }
                    *reinterpret_cast<bf16x8*>(crow + n) = o;
                }
            }
        return;
    }
    if (MODE == 2) {
#pragma unroll
        for (int j = 0; j < NJ / 2; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + fbase[j] + big_group_feature(g, lk);
                if (n < N) {
                    bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float gt = get(j, 4 * g + e), up = get(j + NJ / 2, 4 * g + e);
                        o[e] = (bf16)(silu_fast(gt) * up);
                    }
                    *reinterpret_cast<bf16x4*>(crow + n) = o;
                }
            }
    } else {
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + fbase[j] + big_group_feature(g, lk);
                if (n < N) {
                    bf16x4 o;
                    if (MODE == 1) {
                        const bf16x4 rv = *reinterpret_cast<const bf16x4*>(R + (size_t)m * N + n);
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = (bf16)(get(j, 4 * g + e) + (float)rv[e]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = (bf16)get(j, 4 * g + e);
                    }
                    *reinterpret_cast<bf16x4*>(crow + n) = o;
                }
            }
    }
}

template <int MODE, int NJ, int WN>
__device__ __forceinline__ void big_feature_bases(int wn, int (&fbase)[NJ], int (&wrow)[NJ]) {
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        int row;       // row of the weight tile (0..127 gate / plain, 128..255 up / plain)
        if (MODE == 2) row = (j < NJ / 2) ? (wn * (NJ / 2) + j) * 32 : 128 + (wn * (NJ / 2) + (j - NJ / 2)) * 32;
        else row = (wn * NJ + j) * 32;
        fbase[j] = (MODE == 2 && j >= NJ / 2) ? row - 128 : row;     // output feature offset inside the tile
        wrow[j] = row;
    }
}

// Tile scheduling.  A launch runs one workgroup per CU at a time, so `tiles` whole tiles take
// ceil(tiles / 256) rounds and a last round with few tiles wastes most of the chip.  The first
// n_dp tiles (a multiple of 256) are computed whole by one launch; each of the remaining tiles is
// cut into `splits` ranges of K, one workgroup each (a second launch of the PARTIAL instantiation,
// which starts as the first drains), which write fp32 partial tiles to `ws`; a small third kernel
// adds the partial tiles in range order and applies the epilogue.  The cut is a function of the
// problem shape only.
template <int MODE, int WN, bool PARTIAL>
__global__ __launch_bounds__(128 * WN, 1) void gemm_big_kernel(const bf16* __restrict__ A, const bf16* __restrict__ W,
                                                                const bf16* R, bf16* C, int M, int N, int K,
                                                                int tiles_m, int tiles_n, int n_dp, int splits,
                                                                float* __restrict__ ws) {
    constexpr int NWAVES = 2 * WN;
    constexpr int NJ = 8 / WN;                 // 32-wide feature blocks per wave (gate+up blocks in SwiGLU mode)
    constexpr int NCH = 32 / NWAVES;           // 1 KiB chunks of each tile filled by one wave
    constexpr int NMMA = 4 * NJ;               // MFMAs per k-step
    constexpr int NFETCH = 4 + NJ;             // LDS operand reads per k-step
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];

    const int nk = K / kBK;
    int pid, kt0 = 0, kt1 = nk;
    const int slot = blockIdx.x;                       // PARTIAL: (split tile, K range)
    if (!PARTIAL) {
        pid = xcd_remap(blockIdx.x, n_dp);
    } else {
        pid = n_dp + slot / splits;
        const int per = (nk + splits - 1) / splits;
        kt0 = (slot % splits) * per;
        kt1 = (kt0 + per < nk) ? kt0 + per : nk;
    }
    const BigTile bt = big_tile_of<MODE>(pid, tiles_m, tiles_n);
    const int m0 = bt.m0, n0 = bt.n0;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int lrow = lane & 31, lk = lane >> 5;

    // ---- loader: this wave fills chunks q = wave*NCH + j (rows 8q .. 8q+7) of both tiles.  Addresses
    // are a uniform base (advanced per K tile) plus a per-lane 32-bit byte offset.
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    uint32_t a_off[NCH], b_off[NCH];
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
        const int row = (wave * NCH + j) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ swz(row);
        int ar = m0 + row;
        if (ar > M - 1) ar = M - 1;
        a_off[j] = ((uint32_t)ar * (uint32_t)K + c * 8) * 2u;
        const int frow = (row & ~31) | big_row_feature(row & 31);     // the feature this LDS row holds
        int br;
        if (MODE == 2) {
            const bool up = frow >= 128;
            int f = n0 + (up ? frow - 128 : frow);
            if (f > N - 1) f = N - 1;
            br = up ? N + f : f;
        } else {
            br = n0 + frow;
            if (br > N - 1) br = N - 1;
        }
        b_off[j] = ((uint32_t)br * (uint32_t)K + c * 8) * 2u;
    }
    // Unit u = 2t is the activation half of k-tile t, u = 2t + 1 its weight half; unit u lives in slot
    // u % 5.  Piece q in [0, NCH) of a unit is this wave's q-th 1 KiB chunk.  Past the last k-tile the
    // last one is fetched again (into a slot nobody reads any more) so that every tile issues the
    // same number of loads and the wait counts below hold for every tile.
    // Loads take the buffer form: resource in scalar registers, the lane's byte offset in one vector register,
    // the k-tile's byte offset in a scalar register.  The flat form made the compiler add a 64-bit base to the
    // offset with a vector instruction before every load, and vector ALU instructions in this loop cost matrix
    // time (16 of them per k-tile and wave: 1.3 - 1.5 % of the GEMM).
    const __amdgpu_buffer_rsrc_t rsrc_a =
        __builtin_amdgcn_make_buffer_rsrc((void*)A, 0, (int)((uint32_t)M * (uint32_t)K * 2u), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc(
        (void*)W, 0, (int)((uint32_t)(MODE == 2 ? 2 * N : N) * (uint32_t)K * 2u), 0x00020000);
    auto issue_piece = [&](int kt, int slot, bool weights, int q) {
        unsigned char* sa = smem_raw + slot * kBigSlot + (wave_u * NCH + q) * 1024;
        const int t = kt < kt1 ? kt : kt1 - 1;
        if (!weights) __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (lptr_t)sa, 16, (int)a_off[q], t * (kBK * 2), 0, 0);
        else __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_w, (lptr_t)sa, 16, (int)b_off[q], t * (kBK * 2), 0, 0);
    };
    auto issue_unit = [&](int kt, int slot, bool weights) {
#pragma unroll
        for (int q = 0; q < NCH; ++q) issue_piece(kt, slot, weights, q);
    };

    f32x16 acc[NJ][4];      // [feature block][token block]
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

    // ---- operand addresses inside a stage
    int x_off[4], w_off[NJ], k_off[4], fbase[NJ];
    const int sw = swz(lrow);
#pragma unroll
    for (int i = 0; i < 4; ++i) x_off[i] = (wm * 128 + i * 32 + lrow) * 128;
    {
        int wrow[NJ];
        big_feature_bases<MODE, NJ, WN>(wn, fbase, wrow);
#pragma unroll
        for (int j = 0; j < NJ; ++j) w_off[j] = (wrow[j] + lrow) * 128;
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) k_off[ks] = ((ks * 2 + lk) ^ sw) * 16;

    // ---- main loop.  Every k-step is NMMA MFMAs in a fixed order; between them, one by one, go the
    // LDS reads that fetch the operands of the NEXT k-step (first half of the k-step) and, after every
    // second MFMA of the other half, one global->LDS load (a load behind an MFMA that already has an LDS
    // read behind it makes the next MFMA late: 1-2.5 % on the four projections).  The order is pinned with scheduling barriers so the matrix pipe never waits
    // behind a burst of memory instructions.  The tile barrier sits before the last k-step, whose
    // operands are already in registers; it is a bare s_barrier (the waits are written out here; a
    // full __syncthreads would drain the loads that are meant to stay in flight).
    //
    // The two slots tile i - 1 released at its barrier are refilled as follows: last k-step of tile
    // i - 1 and first of tile i: weights of tile i + 1 (needed first); k-steps 1 and 2 of tile i:
    // activations of tile i + 2.  Before the barrier of tile i everything but those activations must
    // have landed.
    bf16x8 xf[2][4], wf[2][NJ];
    // per-lane part of every operand address, one register per k-step and operand: a fetch then costs one vector
    // add (slot base + this), the 32-row blocks being immediate offsets from it (worth another 0.6 %)
    int xk[4], wk[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        xk[ks] = x_off[0] + k_off[ks];
        wk[ks] = w_off[0] + k_off[ks];
    }
    auto fetch_piece = [&](const unsigned char* sx, const unsigned char* sw_, int ks, int buf, int q) {   // order of first use
        if (q == 0) wf[buf][0] = *reinterpret_cast<const bf16x8*>(sw_ + wk[ks]);
        else if (q <= 4) xf[buf][q - 1] = *reinterpret_cast<const bf16x8*>(sx + xk[ks] + (q - 1) * 4096);
        else wf[buf][q - 4] = *reinterpret_cast<const bf16x8*>(sw_ + wk[ks] + (w_off[q - 4] - w_off[0]));
    };
    constexpr int PER = NCH / 2;                       // loads per wave per k-step
    constexpr int LGAP = (NMMA - NFETCH) / PER;        // MFMAs between two loads of a wave
    static_assert(LGAP >= 1 && LGAP * PER == NMMA - NFETCH, "the loads of a k-step go behind its LDS reads");
    // one k-step: MFMAs from buffer `cur`; fetch k-step `nks` of the tile in slots (sx, sw_) into the
    // other buffer; request pieces p0 .. p0 + PER - 1 of one operand of k-tile `ikt` into slot `islot`
    auto kstep = [&](int cur, const unsigned char* sx, const unsigned char* sw_, int nks, int ikt, int islot, bool iweights,
                     int p0) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < NMMA; ++q) {
            const int j = q >> 2, i = q & 3;
            acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[cur][j], xf[cur][i], acc[j][i], 0, 0, 0);
            if (q < NFETCH) fetch_piece(sx, sw_, nks, cur ^ 1, q);
            if (q >= NFETCH && (q - NFETCH) % LGAP == LGAP - 1) issue_piece(ikt, islot, iweights, p0 + (q - NFETCH) / LGAP);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    if (M > 0x7fffffff / K || 2 * N > 0x7fffffff / K) return;    // 32-bit offsets (checked on the host too)
    const int n = kt1 - kt0;                           // k-tiles of this workgroup, >= 1
    issue_unit(kt0, 0, false);
    issue_unit(kt0, 1, true);
    issue_unit(kt0 + 1, 2, false);
#pragma unroll
    for (int q = 0; q < NCH / 2; ++q) issue_piece(kt0 + 1, 3, true, q);
    static_assert(WN == 2 && NCH == 8, "the hand-written wait counts below assume four waves filling eight chunks each");
    __builtin_amdgcn_s_waitcnt(0x0F7C);                // vmcnt(12): tile kt0 landed
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < NFETCH; ++q) fetch_piece(smem_raw, smem_raw + kBigSlot, 0, 0, q);
    int sa = 0;                                        // slot of the current tile's activations; its weights follow
    for (int i = 0; i < n; ++i) {
        const int sw1 = (sa + 1 >= kBigSlots) ? sa + 1 - kBigSlots : sa + 1;
        const int na = (sa + 2 >= kBigSlots) ? sa + 2 - kBigSlots : sa + 2;      // next tile's slots
        const int nw = (sa + 3 >= kBigSlots) ? sa + 3 - kBigSlots : sa + 3;
        const int fa2 = (sa + 4 >= kBigSlots) ? sa + 4 - kBigSlots : sa + 4;     // where tile i + 2's activations go
        const unsigned char* sx = smem_raw + sa * kBigSlot;
        const unsigned char* sww = smem_raw + sw1 * kBigSlot;
        kstep(0, sx, sww, 1, kt0 + i + 1, nw, true, NCH / 2);
        kstep(1, sx, sww, 2, kt0 + i + 2, fa2, false, 0);
        kstep(0, sx, sww, 3, kt0 + i + 2, fa2, false, NCH / 2);
        // tile i + 1 has landed (only the NCH newest loads, activations of tile i + 2, may be in flight);
        // own LDS reads of tile i are done
        __builtin_amdgcn_s_waitcnt(0x0078);            // vmcnt(8) lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        // tile i + 2's weights, first half, into the slot this tile's activations just left
        kstep(1, smem_raw + na * kBigSlot, smem_raw + nw * kBigSlot, 0, kt0 + i + 2, sa, true, 0);
        sa = na;
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                // no LDS write may be in flight when the workgroup ends

    if (PARTIAL) {
        // partial tile in accumulator order: every (wave, j, i, r) is one 256-byte row of `ws`
        float* base = ws + (size_t)slot * 65536 + (size_t)wave_u * NJ * 4 * 16 * 64;     // wave-uniform
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // a 32-token block wholly past the last row is never read back (a few hundred rows fill
                // only part of a 256-row tile, and the partial tiles are most of the traffic then)
                if (m0 + (wave_u / WN) * 128 + i * 32 < M) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) base[((j * 4 + i) * 16 + r) * 64 + lane] = acc[j][i][r];
                }
                __builtin_amdgcn_sched_barrier(0);     // one block at a time: few registers besides the accumulators are free
            }
        return;
    }
    if (MODE == 1 && (N & 7) == 0) {
        // R may be C itself (the residual stream is updated in place); a lane reads exactly the addresses it
        // writes, so a token block's residual values are fetched together, and the next block's before this
        // block's stores go out (written as load-then-store the loads would queue behind the stores).
        // 16-byte form: registers 8p..8p+7 of feature block j are features 16p + 8*lk + 0..7.
        bf16x8 rv[2][NJ * 2];
        auto load_r = [&](int i, int buf) {
            int m = m0 + wm * 128 + i * 32 + lrow;
            if (m > M - 1) m = M - 1;                   // rows and features past the end: a valid address, value unused
            const bf16* rrow = R + (size_t)m * N;
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    int n = n0 + fbase[j] + 16 * p + 8 * lk;
                    if (n > N - 8) n = N - 8;
                    rv[buf][j * 2 + p] = *reinterpret_cast<const bf16x8*>(rrow + n);
                }
        };
        load_r(0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (i + 1 < 4) load_r(i + 1, (i + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
            const int m = m0 + wm * 128 + i * 32 + lrow;
            if (m < M) {
                bf16* crow = C + (size_t)m * N;
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int p = 0; p < 2; ++p) {
                        const int n = n0 + fbase[j] + 16 * p + 8 * lk;
                        if (n < N) {
                            bf16x8 o;
#pragma unroll
                            for (int e = 0; e < 8; ++e) o[e] = (bf16)(acc[j][i][8 * p + e] + (float)rv[i & 1][j * 2 + p][e]);
                            *reinterpret_cast<bf16x8*>(crow + n) = o;
                        }
                    }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        return;
    }
    // 8-byte form (N not a multiple of 8; a residual is then read element group by element group)
#pragma unroll
    for (int i = 0; i < 4; ++i)
        big_store_block<MODE, NJ>([&](int j, int x) { return acc[j][i][x]; }, m0 + wm * 128 + i * 32 + lrow, n0, fbase,
                                  lk, R, C, M, N);
}

// Adds the partial tiles of one split tile in range order and applies the epilogue.  One wave per
// (wave of the main kernel, feature block j, token block i, piece of the block's 16 registers): a lane sums
// the values behind one output store, 8 consecutive features (registers 8p..8p+7, a 16-byte store) when
// WIDE - rows of N % 8 == 0 features - else 4 (registers 4g..4g+3).  The ranges are taken four at a time,
// then two, then one, every batch's loads going out together; the sums run in range order whatever the
// batching.  Grid (split tiles, units / 4).
template <int MODE, int WN, bool WIDE>
__global__ __launch_bounds__(256) void gemm_big_fixup(const float* __restrict__ ws, const bf16* R, bf16* C, int M,
                                                      int N, int tiles_m, int tiles_n, int n_dp, int splits) {
    constexpr int NJ = 8 / WN;
    constexpr int NJE = (MODE == 2) ? NJ / 2 : NJ;      // output blocks per wave of the main kernel
    constexpr int NV = (MODE == 2) ? 2 : 1;             // accumulator blocks behind one output block
    constexpr int GV = WIDE ? 8 : 4;                    // values per lane and accumulator block
    constexpr int PB = WIDE ? 1 : 2;                    // bits of the piece index
    const int tile = blockIdx.x;
    const BigTile bt = big_tile_of<MODE>(n_dp + tile, tiles_m, tiles_n);
    const int lane = threadIdx.x & 63;
    const int u = blockIdx.y * 4 + (threadIdx.x >> 6);
    const int piece = u & ((1 << PB) - 1), i = (u >> PB) & 3, j = (u >> (PB + 2)) % NJE, wave = (u >> (PB + 2)) / NJE;
    const int wm = wave / WN, wn = wave % WN;
    const int lrow = lane & 31, lk = lane >> 5;
    int fbase[NJ], wrow[NJ];
    big_feature_bases<MODE, NJ, WN>(wn, fbase, wrow);
    int fb = 0;
#pragma unroll
    for (int jj = 0; jj < NJE; ++jj) fb = (jj == j) ? fbase[jj] : fb;
    if (bt.m0 + wm * 128 + i * 32 >= M) return;          // block past the last row: nothing was stored for it
    const int m = bt.m0 + wm * 128 + i * 32 + lrow;
    const int n = bt.n0 + fb + (WIDE ? 16 * piece + 8 * lk : big_group_feature(piece, lk));
    // the residual does not depend on the sums: requested first (rows and features past the end: a valid
    // address, value unused)
    bf16x8 rv8;
    bf16x4 rv4;
    if (MODE == 1) {
        const int mc = m < M ? m : M - 1;
        int nc = n;
        if (nc > N - GV) nc = N - GV;
        if (WIDE) rv8 = *reinterpret_cast<const bf16x8*>(R + (size_t)mc * N + nc);
        else rv4 = *reinterpret_cast<const bf16x4*>(R + (size_t)mc * N + nc);
    }
    float acc[NV][GV];
#pragma unroll
    for (int v = 0; v < NV; ++v)
#pragma unroll
        for (int e = 0; e < GV; ++e) acc[v][e] = 0.f;
    const float* base = ws + (size_t)tile * splits * 65536 + (size_t)wave * NJ * 4 * 16 * 64 + lane;
    auto batch = [&](int s0, auto nb) {
        constexpr int NB = decltype(nb)::value;
        float t[NB][NV][GV];
#pragma unroll
        for (int q = 0; q < NB; ++q)
#pragma unroll
            for (int v = 0; v < NV; ++v)
#pragma unroll
                for (int e = 0; e < GV; ++e)
                    t[q][v][e] = base[(size_t)(s0 + q) * 65536 + (((j + v * (NJ / 2)) * 4 + i) * 16 + GV * piece + e) * 64];
#pragma unroll
        for (int q = 0; q < NB; ++q)
#pragma unroll
            for (int v = 0; v < NV; ++v)
#pragma unroll
                for (int e = 0; e < GV; ++e) acc[v][e] += t[q][v][e];
    };
    int s0 = 0;
    for (; s0 + 4 <= splits; s0 += 4) batch(s0, std::integral_constant<int, 4>());
    if (s0 + 2 <= splits) { batch(s0, std::integral_constant<int, 2>()); s0 += 2; }
    if (s0 < splits) batch(s0, std::integral_constant<int, 1>());
    if (m >= M || n >= N) return;
    float o[GV];
#pragma unroll
    for (int e = 0; e < GV; ++e) {
        if (MODE == 2) o[e] = silu_fast(acc[0][e]) * acc[NV - 1][e];
        else if (MODE == 1) o[e] = acc[0][e] + (float)(WIDE ? rv8[e] : rv4[e]);
        else o[e] = acc[0][e];
    }
    if (WIDE) {
        bf16x8 w;
#pragma unroll
        for (int e = 0; e < 8; ++e) w[e] = (bf16)o[e];
        *reinterpret_cast<bf16x8*>(C + (size_t)m * N + n) = w;
    } else {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (bf16)o[e];
        *reinterpret_cast<bf16x4*>(C + (size_t)m * N + n) = w;
    }
}

struct BigPlan {
    int tiles_m, tiles_n, n_dp, tail, splits;
    size_t ws_bytes;
};

static BigPlan big_plan(int mode, int M, int N, int K) {
    BigPlan p;
    const int out_bn = (mode == 2) ? 128 : 256;
    p.tiles_m = (M + 255) / 256;
    p.tiles_n = (N + out_bn - 1) / out_bn;
    const int tiles = p.tiles_m * p.tiles_n, nk = K / kBK;
    constexpr int kCUs = 256, kMaxTail = 128, kMaxSplits = 16, kMinKt = 4;
    p.n_dp = tiles;
    p.tail = 0;
    p.splits = 1;
    p.ws_bytes = 0;
    const int full = tiles / kCUs * kCUs, rest = tiles - full;
    // rest <= kMaxTail: the last round is at most half full (then two ranges of K per tile fit the chip).
    // full == 0: fewer tiles than CUs altogether (a few hundred rows, or a narrow output); every tile is
    // split, whatever their number, so that a mid-sized batch still puts the whole chip to streaming the
    // weights.
    if (rest > 0 && (rest <= kMaxTail || full == 0)) {
        int sp = kCUs / rest;
        if (sp > kMaxSplits) sp = kMaxSplits;
        if (sp > nk / kMinKt) sp = nk / kMinKt;
        if (sp >= 2) {
            const int per = (nk + sp - 1) / sp;
            sp = (nk + per - 1) / per;               // every range non-empty
            p.n_dp = full;
            p.tail = rest;
            p.splits = sp;
            p.ws_bytes = (size_t)rest * sp * 65536 * sizeof(float);
        }
    }
    return p;
}

static bool big_ok(int M, int N, int K) {
    return M > 64 && K % kBK == 0 && N % 4 == 0 && (uint64_t)M * K < 0x7fffffffull &&
           (uint64_t)2 * N * K < 0x7fffffffull;          // the large-tile kernel uses 32-bit byte offsets / 2
}

// The large-tile kernel needs the CU's whole 160 KiB of LDS; if the runtime does not grant it (asked once per
// instantiation and device) the caller takes the 128x128 kernel instead.
template <int MODE>
static bool big_available() {
    constexpr int LDS = kBigSlots * kBigSlot;
    static LdsLimit whole, partial;
    const bool a = whole.raise(reinterpret_cast<const void*>(gemm_big_kernel<MODE, kBigWN, false>), LDS);
    const bool b = partial.raise(reinterpret_cast<const void*>(gemm_big_kernel<MODE, kBigWN, true>), LDS);
    return a && b;
}

template <int MODE>
static void launch_big(const bf16* a, const bf16* w, const bf16* r, bf16* c, int M, int N, int K, float* ws,
                       size_t ws_bytes, hipStream_t st) {
    constexpr int LDS = kBigSlots * kBigSlot;
    auto kern = gemm_big_kernel<MODE, kBigWN, false>;
    auto kern_part = gemm_big_kernel<MODE, kBigWN, true>;
    BigPlan p = big_plan(MODE, M, N, K);
    if (p.tail > 0 && (ws == nullptr || ws_bytes < p.ws_bytes)) {     // no scratch: every tile whole
        p.n_dp = p.tiles_m * p.tiles_n;
        p.tail = 0;
        p.splits = 1;
    }
    if (p.n_dp > 0)
        hipLaunchKernelGGL(kern, dim3(p.n_dp), dim3(128 * kBigWN), LDS, st, a, w, r, c, M, N, K, p.tiles_m, p.tiles_n,
                           p.n_dp, p.splits, ws);
    if (p.tail > 0) {
        hipLaunchKernelGGL(kern_part, dim3(p.tail * p.splits), dim3(128 * kBigWN), LDS, st, a, w, r, c, M, N, K,
                           p.tiles_m, p.tiles_n, p.n_dp, p.splits, ws);
        constexpr int kUnits = 2 * kBigWN * ((MODE == 2) ? 4 / kBigWN : 8 / kBigWN) * 16;   // waves * blocks * (i, g)
        if ((N & 7) == 0)
            hipLaunchKernelGGL((gemm_big_fixup<MODE, kBigWN, true>), dim3(p.tail, kUnits / 8), dim3(256), 0, st, ws, r, c,
                               M, N, p.tiles_m, p.tiles_n, p.n_dp, p.splits);
        else
            hipLaunchKernelGGL((gemm_big_fixup<MODE, kBigWN, false>), dim3(p.tail, kUnits / 4), dim3(256), 0, st, ws, r, c,
                               M, N, p.tiles_m, p.tiles_n, p.n_dp, p.splits);
    }
}

// ---------------------------------------------------------------------------------------------
// Skinny kernel for decode-sized problems (M <= 256 rows): the weights are read from HBM exactly
// once and that read is the whole cost, so the job is to keep every CU streaming.  Work is cut
// into tiles of 64 * RB weight rows times KSPLIT slices of K (a function of the shape only); each
// workgroup streams its weight slice and the matching activation slice through a ring of LDS
// stages filled by direct global->LDS loads, multiplies with RB 32x32x16 MFMAs per wave and
// k-step, and writes an fp32 partial tile.  A second kernel adds the slices in slice order and
// applies the epilogue, so the result is deterministic.
//
// RB = 1: 64-row tiles, four 16 KiB stages, two workgroups per CU: short streams (small matrices),
// where many small workgroups start and finish faster.
// RB = 2: 128-row tiles, five 24 KiB stages, one workgroup per CU: long streams.  Every tile re-reads
// the activations from L2, which costs about a tenth of the time at 64 rows; twice the rows halve
// that, and the deeper ring keeps 64 KiB of weights in flight per CU instead of 48.  Measured against
// RB = 1 on the decode shapes (64 rows): 8B-GQA down projection 31.4 -> 28.0 us, gate/up unchanged;
// 70B qkv 40.9 -> 37.1, o 36.1 -> 37.8, gate/up 185 -> 168, down 96.5 -> 78.5 us.  (Three stages and
// two workgroups per CU win on some of these shapes and lose on others.)
// ---------------------------------------------------------------------------------------------
// TB = 32-row blocks of activation rows per wave: a workgroup covers 64 * TB rows (64 when the batch
// has no more; 128 beyond, so that 65..128 rows still read every weight once and 129..256 rows twice).
template <int RB, int TB> struct SkCfg {
    static constexpr int kXBytes = 64 * TB * kBK * (int)sizeof(bf16);         // activations of a stage: 8 KiB * TB
    static constexpr int kStage = kXBytes + 64 * RB * kBK * (int)sizeof(bf16);  // + weights 8 KiB * RB
    static constexpr int kStages = (RB == 1 && TB == 1) ? 4 : 5;
    static constexpr int kLds = kStage * kStages;
    static constexpr int kPerCu = kLds * 2 <= 160 * 1024 ? 2 : 1;
    static constexpr int kSlots = 256 * kPerCu;                               // workgroups the chip holds at a time
};
// Weight matrices from this size on count as long streams: RB = 2, and loads with the non-temporal cache
// policy (read once per step; streamed that way a long read runs faster - gate/up of the 8B shape -6 % -
// a short one does not or gets slower).
constexpr size_t kSkStreamBytes = (size_t)64 << 20;

// vmcnt(n) lgkmcnt(0), n < 64
__device__ __forceinline__ constexpr int sk_wait(int n) { return ((n >> 4) << 14) | 0x0070 | (n & 15); }

// GU (gate/up projection): a tile is 32 * RB gate features (weight rows n0..) and the matching up
// features (rows N + n0..), so that with a single k-slice the workgroup holds both factors of
// silu(gate) * up and writes the activation itself (C != nullptr) instead of partial sums.
// NT: the weight loads carry the non-temporal cache policy.
template <bool GU, bool NT, int RB, int TB>
__global__ __launch_bounds__(256, (SkCfg<RB, TB>::kPerCu)) void gemm_skinny_kernel(const bf16* __restrict__ X,
                                                                                   const bf16* __restrict__ W,
                                                                                   float* __restrict__ partial,
                                                                                   bf16* __restrict__ C, int M, int Nrows,
                                                                                   int K, int n_tiles, int kt_per_split,
                                                                                   int rows, int m_blocks, int units) {
    using Cfg = SkCfg<RB, TB>;
    constexpr int kStage = Cfg::kStage, kStages = Cfg::kStages, kXBytes = Cfg::kXBytes;
    constexpr int LPS = 2 * TB + 2 * RB;              // loads per wave and stage
    constexpr int HALF = 32 * RB;                     // rows per wave along the features (GU: rows per factor)
    constexpr int MT = 64 * TB;                       // activation rows per workgroup
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
    // A unit is one (tile, k-slice); with more activation rows than a workgroup covers it is worked on by
    // m_blocks workgroups.  Workgroups are handed to the eight XCDs in turn, so the workgroups of a
    // unit are given ids 8 apart: same XCD, one right after the other, and the weights the first one
    // pulls from HBM are found in that XCD's L2 by the others.
    const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
    const int unit = (seq / m_blocks) * 8 + xcd;
    if (unit >= units) return;
    const int m0 = (seq % m_blocks) * MT;
    const int tile_n = unit % n_tiles, split = unit / n_tiles;
    // `rows` <= 64 * RB weight rows of those the tile has room for are real (GU: rows / 2 of each factor);
    // the launcher picks it so that the grid fills the chip's workgroup slots evenly
    const int tr = GU ? rows >> 1 : rows;             // real rows per factor (GU) or per tile
    const int n0 = tile_n * tr;
    const int Nh = Nrows >> 1;                        // GU: features per factor
    const int nk = K / kBK;
    const int kt0 = split * kt_per_split;
    const int kt1 = (kt0 + kt_per_split < nk) ? kt0 + kt_per_split : nk;
    const int n = kt1 - kt0;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wf = wave >> 1, wt = wave & 1;          // feature half, token half
    const int lrow = lane & 31, lk = lane >> 5;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);

    // loader: 1 KiB chunks of 8 rows; the first 8 * TB chunks of a stage hold the activation rows, the
    // 8 * RB after them the weight rows; this wave fills 2 * TB of the former and 2 * RB of the latter
    uint32_t x_src[2 * TB], w_src[2 * RB];
#pragma unroll
    for (int j = 0; j < 2 * TB; ++j) {
        const int row = (wave * 2 * TB + j) * 8 + (lane >> 3);
        int xr = m0 + row;
        if (xr > M - 1) xr = M - 1;
        x_src[j] = ((uint32_t)xr * (uint32_t)K + ((lane & 7) ^ swz(row)) * 8) * 2u;
    }
#pragma unroll
    for (int j = 0; j < 2 * RB; ++j) {
        const int row = (wave * 2 * RB + j) * 8 + (lane >> 3);
        int wr;
        if (GU) {                                      // rows past the real ones re-read the tile's last row
            int r = row % HALF;
            if (r > tr - 1) r = tr - 1;
            int f = n0 + r;
            if (f > Nh - 1) f = Nh - 1;
            wr = (row / HALF) * Nh + f;
        } else {
            wr = n0 + (row < tr ? row : tr - 1);
            if (wr > Nrows - 1) wr = Nrows - 1;
        }
        w_src[j] = ((uint32_t)wr * (uint32_t)K + ((lane & 7) ^ swz(row)) * 8) * 2u;
    }
    auto issue = [&](int kt, int stage) {
        const char* xk = reinterpret_cast<const char*>(X + (size_t)kt * kBK);
        const char* wk = reinterpret_cast<const char*>(W + (size_t)kt * kBK);
        unsigned char* sb = smem_raw + stage * kStage;
#pragma unroll
        for (int j = 0; j < 2 * TB; ++j)
            __builtin_amdgcn_global_load_lds((gptr_t)(xk + x_src[j]), (lptr_t)(sb + (wave_u * 2 * TB + j) * 1024), 16, 0, 0);
#pragma unroll
        for (int j = 0; j < 2 * RB; ++j)
            __builtin_amdgcn_global_load_lds((gptr_t)(wk + w_src[j]), (lptr_t)(sb + kXBytes + (wave_u * 2 * RB + j) * 1024),
                                             16, 0, NT ? 2 : 0);
    };

    f32x16 acc[RB][TB];
#pragma unroll
    for (int b = 0; b < RB; ++b)
#pragma unroll
        for (int t = 0; t < TB; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[b][t][r] = 0.f;
    const int sw = swz(lrow);
    const int x_off = (wt * 32 * TB + lrow) * 128;
    const int w_off = kXBytes + (wf * HALF + lrow) * 128;

    // Every workgroup would walk its k-tiles in the same order at about the same pace, so that at any moment the
    // whole chip reads the same 128-byte column of thousands of weight rows; when the row pitch is a power of two
    // those addresses differ in their high bits only and crowd onto few memory channels.  A tile therefore starts
    // its walk tile_n / n_tiles of the way in and wraps around (a function of the shape and the tile alone, so
    // the sum order, and with it every output bit, stays fixed).  Measured in the decode loop: gate/up of the 8B
    // shape 50 -> 41 us, output projection of the 70B shape 32 -> 26 us, its QKV 34 -> 32 us; pitches that are
    // no power of two, and walks of fewer than 32 tiles, gain nothing or lose 1-2 % and keep the plain order.
    const int rot = ((K & (K - 1)) == 0 && n >= 32) ? (int)(((long long)tile_n * n) / n_tiles) : 0;
    auto kmap = [&](int j) { const int r = j + rot; return kt0 + (r >= n ? r - n : r); };   // j-th k-tile of the walk
    // prologue: up to kStages - 1 tiles in flight
#pragma unroll
    for (int t = 0; t < kStages - 1; ++t)
        if (n > t) issue(kmap(t), t);
    int cur = 0, nxt = kStages - 1;                  // stage of tile i; stage the tile requested next goes to
    for (int i = 0; i < n; ++i) {
        // tile i must have landed; the tiles requested after it (LPS loads each) may still be in flight
        const int later = (n - 1 - i < kStages - 2) ? n - 1 - i : kStages - 2;
        if (later >= 4) __builtin_amdgcn_s_waitcnt(sk_wait(4 * LPS));
        else if (later == 3) __builtin_amdgcn_s_waitcnt(sk_wait(3 * LPS));
        else if (later == 2) __builtin_amdgcn_s_waitcnt(sk_wait(2 * LPS));
        else if (later == 1) __builtin_amdgcn_s_waitcnt(sk_wait(LPS));
        else __builtin_amdgcn_s_waitcnt(sk_wait(0));
        __builtin_amdgcn_s_barrier();                              // everyone's part landed; the stage of tile i-1 is free
        __builtin_amdgcn_sched_barrier(0);
        if (i + kStages - 1 < n) issue(kmap(i + kStages - 1), nxt);
        const unsigned char* st = smem_raw + cur * kStage;
        nxt = cur;
        cur = (cur + 1 == kStages) ? 0 : cur + 1;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int ko = ((ks * 2 + lk) ^ sw) * 16;
            bf16x8 xf[TB];
#pragma unroll
            for (int t = 0; t < TB; ++t) xf[t] = *reinterpret_cast<const bf16x8*>(st + x_off + t * 32 * 128 + ko);
#pragma unroll
            for (int b = 0; b < RB; ++b) {
                const bf16x8 wfr = *reinterpret_cast<const bf16x8*>(st + w_off + b * 32 * 128 + ko);
#pragma unroll
                for (int t = 0; t < TB; ++t) acc[b][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfr, xf[t], acc[b][t], 0, 0, 0);
            }
        }
    }

    // lane holds, of token block t, token m0 + wt*32*TB + t*32 + lane%32 and, of block b of its wave's rows,
    // features 8g + 4*(lane/32) + 0..3
    if (GU && C != nullptr) {
        // the up-factor waves hand their accumulators to the gate-factor waves (same lane, same
        // token half) through LDS, which is free once everyone has read the last stage
        float* ex = reinterpret_cast<float*>(smem_raw);
        __syncthreads();
        if (wf == 1) {
#pragma unroll
            for (int b = 0; b < RB; ++b)
#pragma unroll
                for (int t = 0; t < TB; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r) ex[(((wt * RB + b) * TB + t) * 16 + r) * 64 + lane] = acc[b][t][r];
        }
        __syncthreads();
        if (wf == 0) {
#pragma unroll
            for (int t = 0; t < TB; ++t) {
                const int m = m0 + wt * 32 * TB + t * 32 + lrow;
                if (m >= M) continue;
#pragma unroll
                for (int b = 0; b < RB; ++b)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int lf = b * 32 + 8 * g + 4 * lk;
                        const int nn = n0 + lf;
                        if (lf < tr && nn < Nh) {
                            bf16x4 w4;
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float o = acc[b][t][4 * g + e];
                                const float u = ex[(((wt * RB + b) * TB + t) * 16 + 4 * g + e) * 64 + lane];
                                w4[e] = (bf16)(silu_fast(o) * u);
                            }
                            *reinterpret_cast<bf16x4*>(C + (size_t)m * Nh + nn) = w4;
                        }
                    }
            }
        }
        return;
    }
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        const int m = m0 + wt * 32 * TB + t * 32 + lrow;
        if (m >= M) continue;
        float* prow = partial + ((size_t)split * M + m) * Nrows;       // partial[split][m][n]
#pragma unroll
        for (int b = 0; b < RB; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int lf = (GU ? 0 : wf * HALF) + b * 32 + 8 * g + 4 * lk;      // feature inside the tile (GU: the factor)
                const int f = n0 + lf;
                const int nn = GU ? wf * Nh + f : f;
                if (lf < tr && f < (GU ? Nh : Nrows))
                    *reinterpret_cast<float4*>(prow + nn) =
                        make_float4(acc[b][t][4 * g], acc[b][t][4 * g + 1], acc[b][t][4 * g + 2], acc[b][t][4 * g + 3]);
            }
    }
}

template <int MODE>
__global__ __launch_bounds__(256) void gemm_skinny_epilogue(const float* __restrict__ partial, const bf16* R, bf16* C,
                                                            int M, int N, int Nrows, int ksplit) {
    const int idx = blockIdx.x * 256 + threadIdx.x;       // one thread per 4 outputs
    const int per_row = N >> 2;
    if (idx >= M * per_row) return;
    const int m = idx / per_row, n = (idx - m * per_row) * 4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f), u = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int k = 0; k < ksplit; ++k) {
        const float* prow = partial + ((size_t)k * M + m) * Nrows;
        const float4 a = *reinterpret_cast<const float4*>(prow + n);
        s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
        if (MODE == 2) {
            const float4 b = *reinterpret_cast<const float4*>(prow + N + n);
            u.x += b.x; u.y += b.y; u.z += b.z; u.w += b.w;
        }
    }
    float o[4] = {s.x, s.y, s.z, s.w};
    if (MODE == 1) {
        const bf16x4 rv = *reinterpret_cast<const bf16x4*>(R + (size_t)m * N + n);
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] += (float)rv[e];
    }
    if (MODE == 2) {
        const float uu[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = silu_fast(o[e]) * uu[e];
    }
    bf16x4 w;
#pragma unroll
    for (int e = 0; e < 4; ++e) w[e] = (bf16)o[e];
    *reinterpret_cast<bf16x4*>(C + (size_t)m * N + n) = w;
}

struct SkinnyPlan {
    int n_tiles, kt_per_split, ksplit, rows, rb, tb, m_blocks;
    size_t ws_bytes;
};

template <int RB, int TB>
static void skinny_plan_rb(SkinnyPlan& p, int Nrows, int nk, int m_blocks) {
    constexpr int kTile = 64 * RB;
    // Units one round hands out.  The long streams fill every workgroup slot of the chip.  The short ones (64-row tiles
    // over at most 64 tokens) aim at one unit per CU although two fit: half as many K slices halve the partial sums
    // written here and re-read by the consumer (8B decode at 64 tokens: qkv 17.7 -> 16.5 us, o 14.8 -> 12.0 us; a
    // target of 128 or 192 units is slower again, 384 and more as well).
    const int kSlots = ((RB == 1 && TB == 1) ? 256 : SkCfg<RB, TB>::kSlots) / m_blocks;
    p.rb = RB;
    p.tb = TB;
    p.m_blocks = m_blocks;
    p.n_tiles = (Nrows + kTile - 1) / kTile;
    int target = kSlots / p.n_tiles;              // aim at filling every workgroup slot once
    if (target < 1) target = 1;
    p.kt_per_split = (nk + target - 1) / target;
    const int min_kt = nk < 4 * RB ? nk : 4 * RB; // keep the ring worth filling
    if (p.kt_per_split < min_kt) p.kt_per_split = min_kt;
    p.ksplit = (nk + p.kt_per_split - 1) / p.kt_per_split;
    // A grid a little short of a multiple of the slots leaves some of them idle for the whole kernel (448
    // workgroups on 512 slots: an eighth of the chip).  Narrower tiles (down to three quarters of the rows,
    // in steps of 8) bring the count up to the multiple; narrower than that, the activations would be
    // re-read by too many tiles.
    p.rows = kTile;
    const int total = p.n_tiles * p.ksplit;
    const int rounds = (total + kSlots - 1) / kSlots;
    const int want_tiles = rounds * kSlots / p.ksplit;
    if (want_tiles > p.n_tiles) {
        const int r = ((Nrows + want_tiles - 1) / want_tiles + 7) / 8 * 8;
        if (r >= kTile * 3 / 4 && r < kTile) {
            p.rows = r;
            p.n_tiles = (Nrows + r - 1) / r;
        }
    }
}

static SkinnyPlan skinny_plan(int M, int N, int K, int mode) {
    SkinnyPlan p;
    const int Nrows = (mode == 2) ? 2 * N : N;
    const int nk = K / kBK;
    const bool stream = (size_t)Nrows * K * sizeof(bf16) >= kSkStreamBytes;
    if (M <= 64) {
        if (stream) skinny_plan_rb<2, 1>(p, Nrows, nk, 1);
        else skinny_plan_rb<1, 1>(p, Nrows, nk, 1);
    } else {
        const int m_blocks = (M + 127) / 128;
        if (stream) skinny_plan_rb<2, 2>(p, Nrows, nk, m_blocks);
        else skinny_plan_rb<1, 2>(p, Nrows, nk, m_blocks);
    }
    p.ws_bytes = (size_t)p.ksplit * M * Nrows * sizeof(float);
    return p;
}

// Beyond 64 rows a workgroup covers 128.  Against the large-tile kernel with every tile split (the four
// projections of the 8B-GQA shape, us): 65 rows 118 / 167, 128 rows 130 / 182, 192 rows 207 / 204,
// 256 rows 215 / 228; with three blocks (384 rows) it loses, 319 / 250.
constexpr int kSkMaxM = 256;
static bool skinny_ok(int M, int N, int K) {
    return M >= 1 && M <= kSkMaxM && K % kBK == 0 && N % 4 == 0 &&
           (uint64_t)2 * N * K < 0x7fffffffull;          // 32-bit byte offsets into the weights (2N rows in gate/up mode)
}

size_t gemm_workspace_bytes(int mode, int M, int N, int K) {
    if (skinny_ok(M, N, K)) return skinny_plan(M, N, K, mode).ws_bytes;
    if (big_ok(M, N, K)) return big_plan(mode, M, N, K).ws_bytes;
    return 0;
}

static bool skinny_applies(int mode, int M, int N, int K, const float* ws, size_t ws_bytes) {
    return skinny_ok(M, N, K) && ws != nullptr && ws_bytes >= skinny_plan(M, N, K, mode).ws_bytes;
}

struct SkinnyArgs {
    const bf16* a; const bf16* w; float* ws; bf16* direct;
    int M, Nrows, K, n_tiles, kt_per_split, rows, m_blocks, units;
};

template <bool GU, bool NT, int RB, int TB>
static void skinny_go(dim3 grid, hipStream_t st, const SkinnyArgs& g) {
    constexpr int lds = SkCfg<RB, TB>::kLds;
    static LdsLimit limit;               // per instantiation: the LDS limit is a per-function setting
    (void)limit.raise(reinterpret_cast<const void*>(gemm_skinny_kernel<GU, NT, RB, TB>), lds);
    hipLaunchKernelGGL((gemm_skinny_kernel<GU, NT, RB, TB>), grid, dim3(256), lds, st, g.a, g.w, g.ws, g.direct, g.M,
                       g.Nrows, g.K, g.n_tiles, g.kt_per_split, g.rows, g.m_blocks, g.units);
}

// Split-K partial sums only: partial[ksplit][M][Nrows] (Nrows = 2N in SwiGLU mode).  The caller
// folds the slices in slice order, either with gemm_skinny_epilogue or fused into the next kernel.
// `c` (gate/up mode only): where the activation goes when one k-slice covers K; then the return value is 0
// and no partial sums are written.
static int launch_skinny_partial(int mode, const bf16* a, const bf16* w, bf16* c, int M, int N, int K, float* ws,
                                 hipStream_t st) {
    const SkinnyPlan p = skinny_plan(M, N, K, mode);
    const int Nrows = (mode == 2) ? 2 * N : N;
    const int units = p.n_tiles * p.ksplit;
    const dim3 grid((units + 7) / 8 * 8 * p.m_blocks);
    bf16* direct = (mode == 2 && p.ksplit == 1) ? c : nullptr;
    const SkinnyArgs args{a, w, ws, direct, M, Nrows, K, p.n_tiles, p.kt_per_split, p.rows, p.m_blocks, units};
    const bool gu = mode == 2;
    if (p.rb == 2 && p.tb == 2) {
        if (gu) skinny_go<true, true, 2, 2>(grid, st, args); else skinny_go<false, true, 2, 2>(grid, st, args);
    } else if (p.rb == 2) {
        if (gu) skinny_go<true, true, 2, 1>(grid, st, args); else skinny_go<false, true, 2, 1>(grid, st, args);
    } else if (p.tb == 2) {
        if (gu) skinny_go<true, false, 1, 2>(grid, st, args); else skinny_go<false, false, 1, 2>(grid, st, args);
    } else {
        if (gu) skinny_go<true, false, 1, 1>(grid, st, args); else skinny_go<false, false, 1, 1>(grid, st, args);
    }
    if (direct) return 0;
    return p.ksplit;
}

int launch_gemm_partial(int mode, const act_t* a, const bf16* w, int M, int N, int K, float* ws, size_t ws_bytes,
                        hipStream_t st) {
    if (M <= 0 || N <= 0 || !skinny_applies(mode, M, N, K, ws, ws_bytes)) return 0;
    return launch_skinny_partial(mode, a, w, nullptr, M, N, K, ws, st);
}

template <int MODE>
static void launch_skinny(const bf16* a, const bf16* w, const bf16* r, bf16* c, int M, int N, int K, float* ws,
                          hipStream_t st) {
    const int ksplit = launch_skinny_partial(MODE, a, w, c, M, N, K, ws, st);
    if (ksplit == 0) return;                          // the kernel wrote the result itself
    const int Nrows = (MODE == 2) ? 2 * N : N;
    const int threads = M * (N >> 2);
    hipLaunchKernelGGL(gemm_skinny_epilogue<MODE>, dim3((threads + 255) / 256), dim3(256), 0, st, ws, r, c, M, N, Nrows,
                       ksplit);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int MODE>
static void launch_cfg(const bf16* a, const bf16* w, const bf16* r, bf16* c, int M, int N, int K, hipStream_t st) {
    constexpr int OUT_BN = (MODE == 2) ? BN / 2 : BN;
    constexpr int LDS = gemm_lds_bytes<BM, BN>();
    auto kern = gemm_kernel<BM, BN, WAVES_M, WAVES_N, MODE>;
    static LdsLimit limit;             // one per instantiation
    (void)limit.raise(reinterpret_cast<const void*>(kern), LDS);
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + OUT_BN - 1) / OUT_BN;
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(WAVES_M * WAVES_N * 64), LDS, st, a, w, r, c, M, N, K,
                       tiles_m, tiles_n);
}

template <int MODE>
static void launch_mode(const bf16* a, const bf16* w, const bf16* r, bf16* c, int M, int N, int K, float* ws,
                        size_t ws_bytes, hipStream_t st) {
    // The kernel and its tiling are a function of the problem shape only, so a layer's result never
    // depends on which range of layers a call covers.
    if (skinny_applies(MODE, M, N, K, ws, ws_bytes)) {
        launch_skinny<MODE>(a, w, r, c, M, N, K, ws, st);
    } else if (M <= 64) {
        launch_cfg<64, 128, 2, 2, MODE>(a, w, r, c, M, N, K, st);
    } else if (big_ok(M, N, K) && big_available<MODE>()) {
        launch_big<MODE>(a, w, r, c, M, N, K, ws, ws_bytes, st);
    } else {
        launch_cfg<128, 128, 2, 2, MODE>(a, w, r, c, M, N, K, st);
    }
}

void launch_gemm(int mode, const act_t* a, const bf16* w, const act_t* r, act_t* c, int M, int N, int K,
                 float* ws, size_t ws_bytes, hipStream_t st) {
    if (M <= 0 || N <= 0) return;
    switch (mode) {
        case 0: launch_mode<0>(a, w, r, c, M, N, K, ws, ws_bytes, st); break;
        case 1: launch_mode<1>(a, w, r, c, M, N, K, ws, ws_bytes, st); break;
        default: launch_mode<2>(a, w, r, c, M, N, K, ws, ws_bytes, st); break;
    }
}

#else  // BZ_FP32_DEBUG: one thread per output element, fp32 FMA chain in k order

template <int MODE>
__global__ __launch_bounds__(256) void gemm_naive_kernel(const float* __restrict__ A, const bf16* __restrict__ W,
                                                         const float* R, float* C, int M, int N, int K) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)M * N) return;
    const int m = (int)(idx / N), n = (int)(idx % N);
    const float* a = A + (size_t)m * K;
    if (MODE == 2) {
        const bf16* wg = W + (size_t)n * K;
        const bf16* wu = W + (size_t)(N + n) * K;
        float g = 0.f, u = 0.f;
        for (int k = 0; k < K; ++k) {
            g = fmaf(a[k], (float)wg[k], g);
            u = fmaf(a[k], (float)wu[k], u);
        }
        C[idx] = g / (1.0f + expf(-g)) * u;
    } else {
        const bf16* w = W + (size_t)n * K;
        float s = 0.f;
        for (int k = 0; k < K; ++k) s = fmaf(a[k], (float)w[k], s);
        if (MODE == 1) s += R[idx];
        C[idx] = s;
    }
}

size_t gemm_workspace_bytes(int, int, int, int) { return 0; }
int launch_gemm_partial(int, const act_t*, const bf16*, int, int, int, float*, size_t, hipStream_t) { return 0; }

void launch_gemm(int mode, const act_t* a, const bf16* w, const act_t* r, act_t* c, int M, int N, int K,
                 float*, size_t, hipStream_t st) {
    if (M <= 0 || N <= 0) return;
    const size_t total = (size_t)M * N;
    const dim3 grid((unsigned)((total + 255) / 256));
    switch (mode) {
        case 0: hipLaunchKernelGGL(gemm_naive_kernel<0>, grid, dim3(256), 0, st, a, w, r, c, M, N, K); break;
        case 1: hipLaunchKernelGGL(gemm_naive_kernel<1>, grid, dim3(256), 0, st, a, w, r, c, M, N, K); break;
        default: hipLaunchKernelGGL(gemm_naive_kernel<2>, grid, dim3(256), 0, st, a, w, r, c, M, N, K); break;
    }
}

#endif

}  // namespace bz
