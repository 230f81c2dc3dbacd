// Causal attention over the KV cache: a tiled MFMA kernel for sequences with several new tokens
// (prefill) and a split-KV kernel plus fixed-order combine for sequences with one (decode).
//
// Cache layout per (layer, slot, kv head): blocks of 32 positions, K piece-major (k_elem_offset), V
// in pieces of 8 positions (v_elem_offset): both are the row-operand order of the 32x32x16 MFMA.
// Query head h reads kv head h / (Hq/Hkv).  A query at absolute position p sees keys 0..p.  Scores
// are scaled by 1/sqrt(d); softmax is evaluated in base 2 (scores pre-multiplied by log2 e).
//
// V is multiplied by probability 0 (not skipped) at masked positions of a partly visible block, so
// cache memory must hold finite values everywhere: the arena is cleared when an instance is created
// and only finite values are ever written by the kernels.
#include "common.h"

namespace bz {

// Loads of cache contents that are read once per step (decode attention): non-temporal, so that the
// stream does not push through the caches what nobody will read again; on this chip a streaming read
// of that kind runs about a quarter faster than a default one.
template <class T>
__device__ __forceinline__ T stream_load(const T* ptr) { return __builtin_nontemporal_load(ptr); }

constexpr float kLog2e = 1.4426950408889634f;

#ifndef BZ_FP32_DEBUG
typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// 2^x by the hardware instruction alone (results below the normal range flush to zero, which is
// what a softmax weight that small should be anyway)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ---------------------------------------------------------------------------------------------
// Prefill.  One workgroup = 128 query rows of one (sequence, head); each of its 4 waves owns 32
// rows.  The wave computes S^T = K * Q^T with 32x32x16 MFMAs, so that a lane (and its partner
// lane + 32) holds all scores of ONE query row: row max / sum need a single cross-lane exchange
// and the running rescale of O^T is a per-lane scalar.  P^T feeds the second MFMA (O^T = V^T *
// P^T) straight from registers: the accumulator layout of S^T is a permutation of the B-operand
// layout along the contraction index, and the V cache stores its pieces in that permuted order.
//
// A KV tile is 64 positions = two cache blocks of K and two of V, each block contiguous in the
// cache in exactly the order the MFMAs read it, so a tile is moved global -> LDS by the DMA path
// (no registers), double-buffered: tile i+1 is in flight while tile i is multiplied.
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256, 2) void attn_prefill_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ out,
                                                              BatchView bv, KvView kv, int Hq, float scale_log2) {
    constexpr int BQ = kPrefillTileQ, BK = 64;
    constexpr int DB = D / 32;           // 32-wide blocks of the head dim
    constexpr int KS = D / 16;           // MFMA k-steps over the head dim
    constexpr int BLK = 32 * D;          // elements per cache block
    constexpr int NL = D / 32;           // 1 KiB DMA loads per wave per tile, for K and again for V
    constexpr int STAGE = 4 * BLK;       // elements per stage: K tile (2 blocks) then V tile (2 blocks)
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16* smem = reinterpret_cast<bf16*>(smem_raw);

    // Workgroups go to the eight XCDs in turn.  With a multiple of 8 heads, XCD x takes Hq / 8 consecutive
    // heads; it walks them kv group by kv group, and inside a group query tile by query tile with the group's
    // heads next to each other: the workgroups that run on an XCD at the same time then read the K and V of
    // one kv head (of a few sequences) and find them in that XCD's L2.  (Dealt out head by head across the
    // XCDs, every L2 fetched every K and V: 2.6 times the algorithmic traffic, and 11 % (MHA) to 21 % (8
    // query heads per kv head) more time.)
    int item, h;
    if ((Hq & 7) == 0) {
        const int xcd = blockIdx.x & 7;
        int seq = blockIdx.x >> 3;
        const int hpx = Hq >> 3, G = Hq / kv.Hkv;
        // A grid that fits the chip's slots in one go (two workgroups per CU, 64 per XCD) lasts as long as its
        // busiest CU.  An XCD's CUs take its workgroups 0..31 first and 32.. as their second one, so CU c holds
        // workgroups c and 32 + c; with the items ordered longest first that pairs long with long.  The second
        // half is therefore walked backwards: CU c gets the c-th longest and the c-th shortest (one 2000-token
        // sequence: 73 -> 60 us).  Larger grids are handed out as slots free up; longest first is right there.
        const int n_x = bv.n_prefill_items * hpx;
        if (n_x <= 64 && seq >= 32) seq = 32 + (n_x - 1 - seq);
        // heads of one kv group that sit next to each other on this XCD (1 if groups do not tile its heads)
        const int gl = G >= hpx ? hpx : (hpx % G == 0 ? G : 1);
        const int per_group = bv.n_prefill_items * gl;
        const int grp = seq / per_group, r = seq - grp * per_group;
        item = r / gl;
        h = xcd * hpx + grp * gl + (r - item * gl);
    } else {
        h = blockIdx.x / bv.n_prefill_items;
        item = blockIdx.x % bv.n_prefill_items;
    }
    const int s = bv.prefill_items[2 * item], qt = bv.prefill_items[2 * item + 1];
    const int q0 = bv.q_start[s];
    const int qlen = bv.q_start[s + 1] - q0;
    const int before = bv.kv_before[s];
    const int slot = bv.seq_slot[s];
    const int Hkv = kv.Hkv;
    const int cap = kv.slot_cap[slot];
    const int kvh = h / (Hq / Hkv);
    const size_t head_base = (size_t)kv.slot_off[slot] * Hkv * D + (size_t)kvh * cap * D;
    const bf16* Kc = kv.k + head_base;
    const bf16* Vc = kv.v + head_base;
    const int nqkv = (Hq + 2 * Hkv) * D;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int lq = lane & 31, lh = lane >> 5;
    const int qi = qt * BQ + wave * 32 + lq;
    const bool valid = qi < qlen;
    const int qic = valid ? qi : qlen - 1;
    const int qpos = before + qic;

    const int last_q = ((qt * BQ + BQ < qlen) ? qt * BQ + BQ : qlen) - 1;
    const int kv_end = before + last_q + 1;                 // keys 0..kv_end-1 are visible to this tile
    const int ntiles = (kv_end + BK - 1) / BK;
    const int last_blk = (kv_end - 1) >> 5;
    int wq_first = qt * BQ + wave * 32, wq_last = wq_first + 31;
    if (wq_last > qlen - 1) wq_last = qlen - 1;
    if (wq_first > qlen - 1) wq_first = qlen - 1;
    const int wave_max_pos = before + wq_last, wave_min_pos = before + wq_first;

    // tile -> LDS: wave w moves 1 KiB pieces w*NL .. w*NL+NL-1 of the K tile and of the V tile.  A
    // block past the last visible one is replaced by the last visible block (its scores are masked).
    // load q in [0, 2*NL) of a tile: K pieces first (needed first), then V pieces
    auto issue_one = [&](int tile, int stage, int q) {
        bf16* st = smem + stage * STAGE;
        const int j = q % NL;
        const int piece = wave_u * NL + j;                   // 512 elements each
        const int blk = piece / (BLK / 512), off = (piece % (BLK / 512)) * 512;
        int kb = tile * 2 + blk;
        if (kb > last_blk) kb = last_blk;
        const size_t src = (size_t)kb * BLK + off + lane * 8;
        if (q < NL) __builtin_amdgcn_global_load_lds((gptr_t)(Kc + src), (lptr_t)(st + piece * 512), 16, 0, 0);
        else __builtin_amdgcn_global_load_lds((gptr_t)(Vc + src), (lptr_t)(st + 2 * BLK + piece * 512), 16, 0, 0);
    };
    auto issue = [&](int tile, int stage) {
#pragma unroll
        for (int q = 0; q < 2 * NL; ++q) issue_one(tile, stage, q);
    };
    issue(0, 0);

    bf16x8 qf[KS];
    {
        const bf16* qp = qkv + (size_t)(q0 + qic) * nqkv + h * D + lh * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
    }

    f32x16 o[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[b][r] = 0.f;
    float m = -INFINITY, l = 0.f;           // running max (already scaled) and sum of this lane's query row

    for (int tile = 0; tile < ntiles; ++tile) {
        const int kbase = tile * BK;
        __builtin_amdgcn_s_waitcnt(0x0070);                  // own pieces of this tile landed, own LDS reads done
        __syncthreads();                                     // everyone's pieces landed; the other stage is free
        // after the last tile the same tile is requested once more into the idle stage: the load schedule
        // then needs no branch between the MFMAs
        const int nxt = tile + 1 < ntiles ? tile + 1 : tile;
        if (kbase > wave_max_pos) {                          // wave-uniform: tile fully masked for this wave
            issue(nxt, (tile + 1) & 1);
        } else {
            const bf16* Ks = smem + (tile & 1) * STAGE;
            const bf16* Vs = Ks + 2 * BLK;
            f32x16 sacc[2];
            // Operand fetch runs ahead of the MFMAs by hand: written as "read, multiply" the compiler waits for
            // every LDS read right before its MFMA, and the score phase takes 2.6 times its 16 MFMAs.  Here the
            // eight K fragments of the first key block are requested together; each is replaced by the second
            // block's fragment as soon as its MFMA has gone, and under the second block's MFMAs the V fragments
            // of the first two k-steps of P.V are requested.
            // The next tile's loads go out one by one between the score MFMAs: a load holds the wave's
            // instruction stream for tens of cycles, which an MFMA in flight covers.
            constexpr int EVERY = (2 * KS) / (2 * NL);
            auto k_frag = [&](int kb, int ks) {
                return *reinterpret_cast<const bf16x8*>(&Ks[kb * BLK + ((ks * 2 + lh) * 32 + lq) * 8]);
            };
            auto v_frag = [&](int t, int b) {
                return *reinterpret_cast<const bf16x8*>(&Vs[(t >> 1) * BLK + ((2 * (t & 1) + lh) * D + b * 32 + lq) * 8]);
            };
            bf16x8 ka[KS], vfr[2][DB];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) ka[ks] = k_frag(0, ks);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) sacc[kb][r] = 0.f;
            __builtin_amdgcn_sched_barrier(0);             // the order below is the order wanted: nothing is moved across
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qf[ks], sacc[kb], 0, 0, 0);
                    if (kb == 0) ka[ks] = k_frag(1, ks);
                    else if (ks < 2 * DB) vfr[ks / DB][ks % DB] = v_frag(ks / DB, ks % DB);
                    const int m = kb * KS + ks;
                    if (m % EVERY == EVERY - 1) issue_one(nxt, (tile + 1) & 1, m / EVERY);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (kbase + BK - 1 > wave_min_pos) {             // wave-uniform: the diagonal crosses this tile
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int kvi = kbase + kb * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                        if (kvi > qpos) sacc[kb][r] = -INFINITY;
                    }
            }
            float mx = -INFINITY;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kb][r]);
            mx = fmaxf(m, mx * scale_log2);                  // scale > 0: max commutes with it
            mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
            if (__builtin_amdgcn_ballot_w64(mx != m) != 0) { // some row's max moved: rescale (wave-uniform)
                const float alpha = fast_exp2(m - mx);       // m = -inf on the first tile -> 0
                l *= alpha;
#pragma unroll
                for (int b = 0; b < DB; ++b)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[b][r] *= alpha;
                m = mx;
            }
            float rs = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float p = fast_exp2(fmaf(sacc[kb][r], scale_log2, -mx));
                    sacc[kb][r] = p;
                    rs += p;
                }
            rs += __shfl_xor(rs, 32, kWave);
            l += rs;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                bf16x8 pf;
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[e] = (bf16)sacc[t >> 1][8 * (t & 1) + e];
#pragma unroll
                for (int b = 0; b < DB; ++b) {
                    o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[t & 1][b], pf, o[b], 0, 0, 0);
                    if (t + 2 < 4) vfr[t & 1][b] = v_frag(t + 2, b);
                }
            }
        }
    }

    __builtin_amdgcn_s_waitcnt(0x0F70);                      // no LDS write may be in flight when the workgroup ends
    if (valid) {
        const float inv = 1.0f / l;
        bf16* op = out + (size_t)(q0 + qi) * Hq * D + h * D;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                bf16x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (bf16)(o[b][r4 * 4 + e] * inv);
                *reinterpret_cast<bf16x4*>(op + b * 32 + 8 * r4 + 4 * lh) = w;
            }
    }
}

template <int D>
static void launch_prefill_d(const act_t* qkv, act_t* out, const BatchView& bv, const KvView& kv, int Hq,
                             hipStream_t st) {
    constexpr int kLds = 2 * 4 * 32 * D * (int)sizeof(bf16);     // two stages of (K tile + V tile)
    static LdsLimit limit;
    (void)limit.raise(reinterpret_cast<const void*>(attn_prefill_kernel<D>), kLds);
    const float scale_log2 = kLog2e / sqrtf((float)D);
    hipLaunchKernelGGL(attn_prefill_kernel<D>, dim3(bv.n_prefill_items * Hq), dim3(256), kLds, st, qkv, out, bv, kv, Hq,
                       scale_log2);
}

void launch_attn_prefill(const act_t* qkv, act_t* out, const BatchView& bv, const KvView& kv, int Hq,
                         hipStream_t st) {
    if (bv.n_prefill_items <= 0) return;
    if (kv.d == 128) launch_prefill_d<128>(qkv, out, bv, kv, Hq, st);
    else launch_prefill_d<64>(qkv, out, bv, kv, Hq, st);
}

#else  // BZ_FP32_DEBUG
// ---------------------------------------------------------------------------------------------
// fp32 debug prefill: one wave per (token, head); scores for all visible keys are kept in LDS and
// softmax is the plain three-pass form.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void attn_naive_kernel(const float* __restrict__ qkv, float* __restrict__ out,
                                                        BatchView bv, KvView kv, int Hq, float scale_log2) {
    extern __shared__ float sc[];
    const int t = blockIdx.x, h = blockIdx.y;
    const int s = bv.token_seq[t];
    if (bv.q_start[s + 1] - bv.q_start[s] <= 1) return;     // single-token sequences use the decode kernel
    const int pos = bv.kv_before[s] + (t - bv.q_start[s]);
    const int slot = bv.seq_slot[s];
    const int D = kv.d, Hkv = kv.Hkv, cap = kv.slot_cap[slot];
    const int kvh = h / (Hq / Hkv);
    const size_t head_base = (size_t)kv.slot_off[slot] * Hkv * D + (size_t)kvh * cap * D;
    const float* Kc = kv.k + head_base;
    const float* Vc = kv.v + head_base;
    const float* q = qkv + (size_t)t * (Hq + 2 * Hkv) * D + h * D;
    const int lane = threadIdx.x;
    float mx = -INFINITY;
    for (int j = lane; j <= pos; j += 64) {
        float a = 0.f;
        for (int e = 0; e < D; ++e) a = fmaf(q[e], Kc[k_elem_offset(j, e, D)], a);
        a *= scale_log2;
        sc[j] = a;
        mx = fmaxf(mx, a);
    }
    mx = wave_max(mx);
    float sum = 0.f;
    for (int j = lane; j <= pos; j += 64) {
        const float p = exp2f(sc[j] - mx);
        sc[j] = p;
        sum += p;
    }
    sum = wave_sum(sum);
    __syncthreads();
    for (int e = lane; e < D; e += 64) {
        float a = 0.f;
        for (int j = 0; j <= pos; ++j) a = fmaf(sc[j], Vc[v_elem_offset(j, e, D)], a);
        out[(size_t)t * Hq * D + h * D + e] = a / sum;
    }
}

void launch_attn_prefill(const act_t* qkv, act_t* out, const BatchView& bv, const KvView& kv, int Hq,
                         hipStream_t st) {
    if (bv.n_prefill_items <= 0) return;
    const float scale_log2 = kLog2e / sqrtf((float)kv.d);
    // 64 KiB of LDS holds 16384 scores: enough for every supported max_seq_len in the debug build
    static LdsLimit limit;
    (void)limit.raise(reinterpret_cast<const void*>(attn_naive_kernel), 65536);
    hipLaunchKernelGGL(attn_naive_kernel, dim3(bv.T, Hq), dim3(64), 65536, st, qkv, out, bv, kv, Hq, scale_log2);
}
#endif

// ---------------------------------------------------------------------------------------------
// Decode.  Grid (chunk, kv head, decode sequence).  A workgroup handles kDecodeChunk = 256 cached
// positions of one kv head for all G = Hq/Hkv query heads that share it: every K and V byte is
// read from HBM once.  Each of the 4 waves owns 64 positions and runs on its own until the four
// partial results are merged.  Each workgroup writes an unnormalised partial (o, running max, sum)
// per head; the combine kernel folds the chunks of a sequence in increasing chunk order, so the
// result does not depend on scheduling.
// ---------------------------------------------------------------------------------------------
#ifndef BZ_FP32_DEBUG
constexpr int kDecodeMaxG = 8;

// Both products run on the matrix cores with the cache as the row operand, read from global
// memory straight into the instructions (a lane's 16 bytes are one operand register pair):
//   S^T[pos, g] = K[pos, :] . q[g, :]     q fills G of the 32 columns, the rest are zero;
//   O^T[j, g]   = V^T[j, pos] . P^T[pos, g]   P^T goes from the score accumulators to the column
//   operand inside the registers (the V cache is stored in the matching position order).
template <int D>
__global__ __launch_bounds__(256, 2) void attn_decode_kernel(const bf16* __restrict__ qkv, float* __restrict__ partial,
                                                             BatchView bv, KvView kv, int Hq, int G, float scale_log2) {
    constexpr int CH = kDecodeChunk;
    constexpr int KS = D / 16, DB = D / 32, BLK = 32 * D;
    __shared__ float wmx[4][kDecodeMaxG];
    __shared__ float wsum[4][kDecodeMaxG];
    __shared__ float osh[4][kDecodeMaxG][D];

    // the work list names only chunks that exist, and brings the sequence's slot along: everything else
    // hangs off one more level of loads (see BatchView for the order of workgroups)
    const int e = blockIdx.x / kv.Hkv;
    const int4 item = bv.decode_work[2 * e], item2 = bv.decode_work[2 * e + 1];
    const int s = item.x, slot = item.y, di = item.z;
    const int rest = blockIdx.x - kv.Hkv * item2.x;          // position among this sequence's (kv head, chunk) pairs
    const int kvh = rest / item.w, chunk = rest - kvh * item.w;
    const int len = bv.kv_before[s] + 1;
    const int c0 = chunk * CH;
    if (c0 >= len) return;
    const int t = bv.q_start[s];
    const int Hkv = kv.Hkv, cap = kv.slot_cap[slot];
    const size_t head_base = (size_t)kv.slot_off[slot] * Hkv * D + (size_t)kvh * cap * D;
    const bf16* Kc = kv.k + head_base;
    const bf16* Vc = kv.v + head_base;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lq = lane & 31, lh = lane >> 5;
    const bf16* q = qkv + (size_t)t * (Hq + 2 * Hkv) * D + (size_t)kvh * G * D;    // G query heads, contiguous

    const int w0 = c0 + wave * 64;
    if (w0 < len) {                                          // wave-uniform
        const int last_blk = (len - 1) >> 5;
        // a block past the end is replaced by the last valid one (loads stay unconditional and in
        // bounds); its positions get probability zero
        size_t boff[2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            int kb = (w0 >> 5) + rb;
            if (kb > last_blk) kb = last_blk;
            boff[rb] = (size_t)kb * BLK;
        }
        bf16x8 kf[2][KS], vf[2][2][DB];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                kf[rb][ks] = stream_load(reinterpret_cast<const bf16x8*>(Kc + boff[rb] + ((ks * 2 + lh) * 32 + lq) * 8));
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                for (int db = 0; db < DB; ++db)
                    vf[rb][tt][db] =
                        stream_load(reinterpret_cast<const bf16x8*>(Vc + boff[rb] + ((2 * tt + lh) * D + db * 32 + lq) * 8));
        bf16x8 qf[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (lq < G) qf[ks] = *reinterpret_cast<const bf16x8*>(q + lq * D + ks * 16 + lh * 8);
            else
#pragma unroll
                for (int e = 0; e < 8; ++e) qf[ks][e] = (bf16)0.f;
        }
        f32x16 sacc[2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[rb][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                sacc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[rb][ks], qf[ks], sacc[rb], 0, 0, 0);
        }
        // lane (g = lane%32, h = lane/32) holds positions rb*32 + 8*(r/4) + 4h + r%4 of head g
        float m = -INFINITY;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int pl = rb * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                const float sg = (w0 + pl < len) ? sacc[rb][r] * scale_log2 : -INFINITY;
                sacc[rb][r] = sg;
                m = fmaxf(m, sg);
            }
        m = fmaxf(m, __shfl_xor(m, 32, kWave));              // finite: position w0 is valid
        float l = 0.f;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = exp2f(sacc[rb][r] - m);
                sacc[rb][r] = p;
                l += p;
            }
        l += __shfl_xor(l, 32, kWave);
        f32x16 oacc[DB];
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                bf16x8 pf;
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[e] = (bf16)sacc[rb][8 * tt + e];
#pragma unroll
                for (int db = 0; db < DB; ++db)
                    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[rb][tt][db], pf, oacc[db], 0, 0, 0);
            }
        if (lq < G) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4)
                    *reinterpret_cast<float4*>(&osh[wave][lq][db * 32 + 8 * r4 + 4 * lh]) =
                        make_float4(oacc[db][4 * r4], oacc[db][4 * r4 + 1], oacc[db][4 * r4 + 2], oacc[db][4 * r4 + 3]);
            if (lh == 0) {
                wmx[wave][lq] = m;
                wsum[wave][lq] = l;
            }
        }
    } else {                                                 // nothing cached in this wave's range
        for (int i = lane; i < G * D; i += 64) osh[wave][i / D][i % D] = 0.f;
        if (lane < G) {
            wmx[wave][lane] = -INFINITY;
            wsum[wave][lane] = 0.f;
        }
    }
    __syncthreads();
    // merge the four waves in wave order
    const int PS = decode_partial_stride(D);
    for (int i = tid; i < G * D; i += 256) {
        const int g = i / D, dd = i - g * D;
        const float M = fmaxf(fmaxf(wmx[0][g], wmx[1][g]), fmaxf(wmx[2][g], wmx[3][g]));
        float acc = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) acc = fmaf(osh[w][g][dd], exp2f(wmx[w][g] - M), acc);
        partial[(((size_t)di * Hq + kvh * G + g) * bv.decode_chunks + chunk) * PS + dd] = acc;
    }
    if (tid < G) {
        const int g = tid;
        const float M = fmaxf(fmaxf(wmx[0][g], wmx[1][g]), fmaxf(wmx[2][g], wmx[3][g]));
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) L = fmaf(wsum[w][g], exp2f(wmx[w][g] - M), L);
        float* pp = partial + (((size_t)di * Hq + kvh * G + g) * bv.decode_chunks + chunk) * PS;
        pp[D] = M;
        pp[D + 1] = L;
    }
}

#else
// fp32 debug build: scores with one lane per position, PV with D/8 lanes per position, on the VALU.
template <int D, int G>
__global__ __launch_bounds__(256) void attn_decode_kernel(const float* __restrict__ qkv, float* __restrict__ partial,
                                                          BatchView bv, KvView kv, int Hq, int, float scale_log2) {
    constexpr int CH = kDecodeChunk;
    constexpr int LPR = D / 8;            // lanes per position in the PV product
    constexpr int RPI = 64 / LPR;         // positions per wave step
    constexpr int NSTEP = 64 / RPI;       // steps for the wave's 64 positions
    __shared__ float ps[4][G][64];
    __shared__ float wmx[4][G];
    __shared__ float wsum[4][G];
    __shared__ float osh[4][G][D];
    __shared__ float qs[G][D];

    // the work list names only chunks that exist, and brings the sequence's slot along: everything else
    // hangs off one more level of loads (see BatchView for the order of workgroups)
    const int e = blockIdx.x / kv.Hkv;
    const int4 item = bv.decode_work[2 * e], item2 = bv.decode_work[2 * e + 1];
    const int s = item.x, slot = item.y, di = item.z;
    const int rest = blockIdx.x - kv.Hkv * item2.x;          // position among this sequence's (kv head, chunk) pairs
    const int kvh = rest / item.w, chunk = rest - kvh * item.w;
    const int len = bv.kv_before[s] + 1;
    const int c0 = chunk * CH;
    if (c0 >= len) return;
    const int t = bv.q_start[s];
    const int Hkv = kv.Hkv, cap = kv.slot_cap[slot];
    const size_t head_base = (size_t)kv.slot_off[slot] * Hkv * D + (size_t)kvh * cap * D;
    const float* Kc = kv.k + head_base;
    const float* Vc = kv.v + head_base;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* q = qkv + (size_t)t * (Hq + 2 * Hkv) * D + (size_t)kvh * G * D;
    const int w0 = c0 + wave * 64;
    const int sub = lane / LPR, dv = (lane % LPR) * 8;
    {
        for (int i = tid; i < G * D / 8; i += 256) {
            float v[8];
            load8(q + i * 8, v);
#pragma unroll
            for (int e = 0; e < 8; ++e) (&qs[0][0])[i * 8 + e] = v[e];
        }
        __syncthreads();
        const int pos = w0 + lane;
        const bool valid = pos < len;
        const int kpos = valid ? pos : len - 1;
        float sc[G];
#pragma unroll
        for (int g = 0; g < G; ++g) sc[g] = 0.f;
        for (int c = 0; c < D / 8; ++c) {
            float kk[8];
            load8(Kc + k_piece_offset(kpos, c, D), kk);
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int e = 0; e < 8; ++e) sc[g] = fmaf(kk[e], qs[g][c * 8 + e], sc[g]);
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float sg = valid ? sc[g] * scale_log2 : -INFINITY;
            const float m = wave_max(sg);
            const float p = valid ? exp2f(sg - m) : 0.f;
            ps[wave][g][lane] = p;
            const float l = wave_sum(p);
            if (lane == 0) {
                wmx[wave][g] = m;
                wsum[wave][g] = l;
            }
        }
    }

    float o[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) o[g][e] = 0.f;
    for (int stp = 0; stp < NSTEP; ++stp) {
        const int prow = stp * RPI + sub;
        int vp = w0 + prow;
        if (vp > len - 1) vp = len - 1;                  // probability zero there
        float vf[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) vf[e] = Vc[v_elem_offset(vp, dv + e, D)];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float pw = ps[wave][g][prow];           // written by this wave only
#pragma unroll
            for (int e = 0; e < 8; ++e) o[g][e] = fmaf(pw, vf[e], o[g][e]);
        }
    }
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = o[g][e];
#pragma unroll
            for (int off = LPR; off < 64; off <<= 1) v += __shfl_xor(v, off, kWave);
            o[g][e] = v;
        }
    if (lane < LPR) {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int e = 0; e < 8; ++e) osh[wave][g][dv + e] = o[g][e];
    }
    __syncthreads();
    // merge the four waves in wave order
    const int PS = decode_partial_stride(D);
    for (int i = tid; i < G * D; i += 256) {
        const int g = i / D, dd = i - g * D;
        const float M = fmaxf(fmaxf(wmx[0][g], wmx[1][g]), fmaxf(wmx[2][g], wmx[3][g]));
        float acc = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) acc = fmaf(osh[w][g][dd], exp2f(wmx[w][g] - M), acc);
        partial[(((size_t)di * Hq + kvh * G + g) * bv.decode_chunks + chunk) * PS + dd] = acc;
    }
    if (tid < G) {
        const int g = tid;
        const float M = fmaxf(fmaxf(wmx[0][g], wmx[1][g]), fmaxf(wmx[2][g], wmx[3][g]));
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) L = fmaf(wsum[w][g], exp2f(wmx[w][g] - M), L);
        float* pp = partial + (((size_t)di * Hq + kvh * G + g) * bv.decode_chunks + chunk) * PS;
        pp[D] = M;
        pp[D + 1] = L;
    }
}

#endif

// One workgroup per (decode sequence, head), one thread per head-dim index.  Chunks are folded in
// increasing order, sixteen per batch: all loads of a batch are independent (an index past the end
// re-reads the last chunk; its value is not added), so a sequence of up to 4096 positions costs one
// memory round trip.  Across batches the running (max, numerator, denominator) is rescaled.
template <int D>
__global__ __launch_bounds__(D) void attn_combine_kernel(const float* __restrict__ partial, act_t* __restrict__ out,
                                                         BatchView bv, int Hq) {
    constexpr int NB = 16;
    const int di = blockIdx.x, h = blockIdx.y, dd = threadIdx.x;
    const int s = bv.decode_seqs[di];
    const int len = bv.kv_before[s] + 1;
    const int nch = (len + kDecodeChunk - 1) / kDecodeChunk;
    const int PS = decode_partial_stride(D);
    const float* base = partial + ((size_t)di * Hq + h) * bv.decode_chunks * PS;
    float M = -INFINITY, num = 0.f, den = 0.f;
    for (int c0 = 0; c0 < nch; c0 += NB) {
        float mv[NB], ov[NB], lv[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const float* pc = base + ((c0 + u < nch) ? c0 + u : nch - 1) * PS;
            mv[u] = pc[D];
            ov[u] = pc[dd];
            lv[u] = pc[D + 1];
        }
        float Mb = M;
#pragma unroll
        for (int u = 0; u < NB; ++u) Mb = fmaxf(Mb, mv[u]);
        const float keep = exp2f(M - Mb);                // 0 for the first batch (M = -inf)
        num *= keep;
        den *= keep;
        M = Mb;
        // no branches here: behind one the compiler moves each load next to its use and the batch turns
        // into sixteen round trips.  A chunk past the end gets weight zero and adds exactly nothing.
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const float w = (c0 + u < nch) ? exp2f(mv[u] - M) : 0.f;
            num = fmaf(ov[u], w, num);
            den = fmaf(lv[u], w, den);
        }
    }
    act_t r;
    from_f32(r, num / den);
    out[(size_t)bv.q_start[s] * Hq * D + h * D + dd] = r;
}

template <int D>
static void launch_decode_d(const act_t* qkv, act_t* out, float* partial, const BatchView& bv, const KvView& kv,
                            int Hq, hipStream_t st) {
    const float scale_log2 = kLog2e / sqrtf((float)D);
    const dim3 grid(bv.n_decode_work * kv.Hkv);
    const int G = Hq / kv.Hkv;                      // 1, 2, 4 or 8: checked when the instance is created
#ifndef BZ_FP32_DEBUG
    hipLaunchKernelGGL(attn_decode_kernel<D>, grid, dim3(256), 0, st, qkv, partial, bv, kv, Hq, G, scale_log2);
#else
    switch (G) {
        case 1: hipLaunchKernelGGL((attn_decode_kernel<D, 1>), grid, dim3(256), 0, st, qkv, partial, bv, kv, Hq, G, scale_log2); break;
        case 2: hipLaunchKernelGGL((attn_decode_kernel<D, 2>), grid, dim3(256), 0, st, qkv, partial, bv, kv, Hq, G, scale_log2); break;
        case 4: hipLaunchKernelGGL((attn_decode_kernel<D, 4>), grid, dim3(256), 0, st, qkv, partial, bv, kv, Hq, G, scale_log2); break;
        default: hipLaunchKernelGGL((attn_decode_kernel<D, 8>), grid, dim3(256), 0, st, qkv, partial, bv, kv, Hq, G, scale_log2); break;
    }
#endif
    hipLaunchKernelGGL(attn_combine_kernel<D>, dim3(bv.n_decode, Hq), dim3(D), 0, st, partial, out, bv, Hq);
}

void launch_attn_decode(const act_t* qkv, act_t* out, float* partial, const BatchView& bv, const KvView& kv,
                        int Hq, hipStream_t st) {
    if (bv.n_decode <= 0) return;
    if (kv.d == 128) launch_decode_d<128>(qkv, out, partial, bv, kv, Hq, st);
    else launch_decode_d<64>(qkv, out, partial, bv, kv, Hq, st);
}

}  // namespace bz
