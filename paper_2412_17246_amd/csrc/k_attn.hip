// Causal attention over the KV cache: a tiled MFMA kernel for sequences with several new tokens
// (prefill) and a split-KV kernel plus fixed-order combine for sequences with one (decode).
//
// Cache layout per (layer, slot, kv head): V[pos][d]; K in blocks of 32 positions stored piece-major
// (k_piece_offset), which is the MFMA row-operand order.  Query head h reads kv head h / (Hq/Hkv).  A query at absolute position p sees keys 0..p.  Scores are scaled by
// 1/sqrt(d); softmax is evaluated in base 2 (scores pre-multiplied by log2 e).
#include "common.h"

namespace bz {

constexpr float kLog2e = 1.4426950408889634f;

#ifndef BZ_FP32_DEBUG
// ---------------------------------------------------------------------------------------------
// Prefill.  One workgroup = 128 query rows of one (sequence, head); each of its 4 waves owns 32
// rows.  The wave computes S^T = K * Q^T with 32x32x16 MFMAs, so that a lane (and its partner
// lane + 32) holds all scores of ONE query row: row max / sum need a single cross-lane exchange
// and the running rescale of O^T is a per-lane scalar.  P^T feeds the second MFMA (O^T = V^T *
// P^T) straight from registers: the accumulator layout of S^T is a permutation of the B-operand
// layout along the contraction index, and V^T is read from LDS with the same permutation.
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void attn_prefill_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ out,
                                                           BatchView bv, KvView kv, int Hq, float scale_log2) {
    constexpr int BQ = kPrefillTileQ, BK = 64;
    constexpr int VROW = BK + 8;     // padded LDS rows (elements)
    constexpr int DB = D / 32;       // 32-wide blocks of the head dim
    constexpr int KS = D / 16;       // MFMA k-steps over the head dim
    __shared__ __attribute__((aligned(16))) bf16 Ks[BK * D];      // two 32-position blocks, piece-major as in the cache
    __shared__ __attribute__((aligned(16))) bf16 Vt[D * VROW];

    const int item = blockIdx.x, h = blockIdx.y;
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
    const int lq = lane & 31, lh = lane >> 5;
    const int qi = qt * BQ + wave * 32 + lq;
    const bool valid = qi < qlen;
    const int qic = valid ? qi : qlen - 1;
    const int qpos = before + qic;

    bf16x8 qf[KS];
    {
        const bf16* qp = qkv + (size_t)(q0 + qic) * nqkv + h * D + lh * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
    }

    const int last_q = ((qt * BQ + BQ < qlen) ? qt * BQ + BQ : qlen) - 1;
    const int kv_end = before + last_q + 1;                 // keys 0..kv_end-1 are visible to this tile
    const int ntiles = (kv_end + BK - 1) / BK;
    int wq_last = qt * BQ + wave * 32 + 31;
    if (wq_last > qlen - 1) wq_last = qlen - 1;
    const int wave_max_pos = before + wq_last;

    f32x16 o[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[b][r] = 0.f;
    float m = -INFINITY, l = 0.f;

    for (int tile = 0; tile < ntiles; ++tile) {
        const int kbase = tile * BK;
        __syncthreads();                                     // all waves are done with the previous tile
        {   // K tile: two 32-position blocks copied as they lie in the cache (a block past the last
            // visible key is replaced by the last visible block; its scores are masked anyway)
            constexpr int VPB = 32 * D / 8;                  // 16-byte vectors per block
#pragma unroll
            for (int p = 0; p < 2 * VPB / 256; ++p) {
                const int v = tid + p * 256;
                const int blk = v / VPB, off = v % VPB;
                int kb = (kbase >> 5) + blk;
                if (kb > ((kv_end - 1) >> 5)) kb = (kv_end - 1) >> 5;
                *reinterpret_cast<uint4*>(&Ks[v * 8]) =
                    *reinterpret_cast<const uint4*>(Kc + (size_t)kb * 32 * D + off * 8);
            }
        }
        {   // V tile, transposed into Vt[d][kv]
            constexpr int CH = D / 8;
#pragma unroll
            for (int p = 0; p < CH / 4; ++p) {
                const int kr = tid & 63, c = (tid >> 6) + 4 * p;
                int kp = kbase + kr;
                if (kp > kv_end - 1) kp = kv_end - 1;
                const bf16x8 v = *reinterpret_cast<const bf16x8*>(Vc + (size_t)kp * D + c * 8);
#pragma unroll
                for (int e = 0; e < 8; ++e) Vt[(c * 8 + e) * VROW + kr] = v[e];
            }
        }
        __syncthreads();
        if (kbase <= wave_max_pos) {                         // wave-uniform: tile not fully masked for this wave
            f32x16 sacc[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int r = 0; r < 16; ++r) sacc[kb][r] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8*>(&Ks[kb * 32 * D + ((ks * 2 + lh) * 32 + lq) * 8]);
                    sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], sacc[kb], 0, 0, 0);
                }
            }
            float mx = m;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kvi = kbase + kb * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                    float sc = sacc[kb][r] * scale_log2;
                    if (kvi > qpos) sc = -INFINITY;
                    sacc[kb][r] = sc;
                    mx = fmaxf(mx, sc);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
            const float alpha = exp2f(m - mx);               // m = -inf on the first tile -> 0
            float rs = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float p = exp2f(sacc[kb][r] - mx);
                    sacc[kb][r] = p;
                    rs += p;
                }
            rs += __shfl_xor(rs, 32, kWave);
            l = l * alpha + rs;
            m = mx;
#pragma unroll
            for (int b = 0; b < DB; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[b][r] *= alpha;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                bf16x8 pf;
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[e] = (bf16)sacc[t >> 1][8 * (t & 1) + e];
#pragma unroll
                for (int b = 0; b < DB; ++b) {
                    const bf16* vp = &Vt[(b * 32 + lq) * VROW + t * 16 + 4 * lh];
                    const bf16x4 v0 = *reinterpret_cast<const bf16x4*>(vp);
                    const bf16x4 v1 = *reinterpret_cast<const bf16x4*>(vp + 8);
                    bf16x8 vf;
                    vf[0] = v0[0]; vf[1] = v0[1]; vf[2] = v0[2]; vf[3] = v0[3];
                    vf[4] = v1[0]; vf[5] = v1[1]; vf[6] = v1[2]; vf[7] = v1[3];
                    o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, o[b], 0, 0, 0);
                }
            }
        }
    }

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

void launch_attn_prefill(const act_t* qkv, act_t* out, const BatchView& bv, const KvView& kv, int Hq,
                         hipStream_t st) {
    if (bv.n_prefill_items <= 0) return;
    const float scale_log2 = kLog2e / sqrtf((float)kv.d);
    const dim3 grid(bv.n_prefill_items, Hq);
    if (kv.d == 128) {
        hipLaunchKernelGGL(attn_prefill_kernel<128>, grid, dim3(256), 0, st, qkv, out, bv, kv, Hq, scale_log2);
    } else {
        hipLaunchKernelGGL(attn_prefill_kernel<64>, grid, dim3(256), 0, st, qkv, out, bv, kv, Hq, scale_log2);
    }
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
        for (int j = 0; j <= pos; ++j) a = fmaf(sc[j], Vc[(size_t)j * D + e], a);
        out[(size_t)t * Hq * D + h * D + e] = a / sum;
    }
}

void launch_attn_prefill(const act_t* qkv, act_t* out, const BatchView& bv, const KvView& kv, int Hq,
                         hipStream_t st) {
    if (bv.n_prefill_items <= 0) return;
    const float scale_log2 = kLog2e / sqrtf((float)kv.d);
    // 64 KiB of LDS holds 16384 scores: enough for every supported max_seq_len in the debug build
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(attn_naive_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
        attr_set = true;
    }
    hipLaunchKernelGGL(attn_naive_kernel, dim3(bv.T, Hq), dim3(64), 65536, st, qkv, out, bv, kv, Hq, scale_log2);
}
#endif

// ---------------------------------------------------------------------------------------------
// Decode.  Grid (chunk, kv head, decode sequence).  A workgroup handles kDecodeChunk = 256 cached
// positions of one kv head for all G = Hq/Hkv query heads that share it: every K and V byte is
// read from HBM once.  Scores: one lane per position (the lane walks its K row in 16-byte steps).
// PV: D/8 lanes per V row, so a wave reads whole rows with 16-byte loads.  Each workgroup writes
// an unnormalised partial (o, running max, sum) per head; the combine kernel folds the chunks of
// a sequence in increasing chunk order, so the result does not depend on scheduling.
// ---------------------------------------------------------------------------------------------
template <int D, int G>
__global__ __launch_bounds__(256) void attn_decode_kernel(const act_t* __restrict__ qkv, float* __restrict__ partial,
                                                          BatchView bv, KvView kv, int Hq, float scale_log2) {
    constexpr int CH = kDecodeChunk;
    constexpr int LPR = D / 8;            // lanes per V row
    constexpr int RPI = 64 / LPR;         // V rows per wave load
    constexpr int NSTEP = 64 / RPI;       // V loads per lane for the wave's 64 positions
    __shared__ float ps[4][G][64];
    __shared__ float wmx[4][G];
    __shared__ float wsum[4][G];
    __shared__ float osh[4][G][D];
#ifdef BZ_FP32_DEBUG
    __shared__ float qs[G][D];
#endif

    const int chunk = blockIdx.x, kvh = blockIdx.y, di = blockIdx.z;
    const int s = bv.decode_seqs[di];
    const int len = bv.kv_before[s] + 1;
    const int c0 = chunk * CH;
    if (c0 >= len) return;
    const int t = bv.q_start[s];
    const int slot = bv.seq_slot[s];
    const int Hkv = kv.Hkv, cap = kv.slot_cap[slot];
    const size_t head_base = (size_t)kv.slot_off[slot] * Hkv * D + (size_t)kvh * cap * D;
    const act_t* Kc = kv.k + head_base;
    const act_t* Vc = kv.v + head_base;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const act_t* q = qkv + (size_t)t * (Hq + 2 * Hkv) * D + (size_t)kvh * G * D;    // G query heads, contiguous

    // Each wave owns 64 positions and runs on its own: no workgroup barrier until the four partial
    // results are merged.  Rows past the end are read from the last valid row (so all loads are
    // unconditional and in bounds) and get probability zero.
    const int w0 = c0 + wave * 64;
    const int sub = lane / LPR, dv = (lane % LPR) * 8;
    raw8_act vv[NSTEP];
#pragma unroll
    for (int stp = 0; stp < NSTEP; ++stp) {           // V rows first: they stay in flight under the score math
        int vp = w0 + stp * RPI + sub;
        if (vp > len - 1) vp = len - 1;
        load_raw8(Vc + (size_t)vp * D + dv, vv[stp]);
    }

#ifndef BZ_FP32_DEBUG
    // Scores on the matrix cores: S^T[pos, g] = K[pos, :] . q[g, :].  A K row is the MFMA's row
    // operand exactly as it lies in memory (lane = position, 16 bytes per k-step), so it goes from
    // global memory straight into the instruction; q fills G of the 32 columns, the rest are zero.
    {
        const int lq = lane & 31, lh = lane >> 5;
        bf16x8 qf[D / 16];
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
            if (lq < G) qf[ks] = *reinterpret_cast<const bf16x8*>(q + lq * D + ks * 16 + lh * 8);
            else
#pragma unroll
                for (int e = 0; e < 8; ++e) qf[ks][e] = (bf16)0.f;
        }
        f32x16 sacc[2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            int kb = (w0 >> 5) + rb;                         // 32-position block; past the end: the last valid one
            if (kb > ((len - 1) >> 5)) kb = (len - 1) >> 5;
            const bf16* kr = Kc + (size_t)kb * 32 * D + (lh * 32 + lq) * 8;
            bf16x8 kf[D / 16];
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) kf[ks] = *reinterpret_cast<const bf16x8*>(kr + ks * 2 * 32 * 8);
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[rb][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks)
                sacc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[ks], sacc[rb], 0, 0, 0);
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
        m = fmaxf(m, __shfl_xor(m, 32, kWave));
        float l = 0.f;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = (sacc[rb][r] == -INFINITY) ? 0.f : exp2f(sacc[rb][r] - m);
                sacc[rb][r] = p;
                l += p;
            }
        l += __shfl_xor(l, 32, kWave);
        if (lq < G) {
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4)
                    *reinterpret_cast<float4*>(&ps[wave][lq][rb * 32 + 8 * r4 + 4 * lh]) =
                        make_float4(sacc[rb][4 * r4], sacc[rb][4 * r4 + 1], sacc[rb][4 * r4 + 2], sacc[rb][4 * r4 + 3]);
            if (lh == 0) {
                wmx[wave][lq] = m;
                wsum[wave][lq] = l;
            }
        }
    }
#else
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
#endif

    float o[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) o[g][e] = 0.f;
#pragma unroll
    for (int stp = 0; stp < NSTEP; ++stp) {
        const int prow = stp * RPI + sub;
        float vf[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) vf[e] = raw_get(vv[stp], e);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float pw = ps[wave][g][prow];       // written by this wave only
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

template <int D>
__global__ __launch_bounds__(D) void attn_combine_kernel(const float* __restrict__ partial, act_t* __restrict__ out,
                                                         BatchView bv, int Hq) {
    const int di = blockIdx.x, h = blockIdx.y, dd = threadIdx.x;
    const int s = bv.decode_seqs[di];
    const int len = bv.kv_before[s] + 1;
    const int nch = (len + kDecodeChunk - 1) / kDecodeChunk;
    const int PS = decode_partial_stride(D);
    const float* base = partial + ((size_t)di * Hq + h) * bv.decode_chunks * PS;
    float M = -INFINITY;
    for (int c = 0; c < nch; ++c) M = fmaxf(M, base[c * PS + D]);
    float num = 0.f, den = 0.f;
    for (int c = 0; c < nch; ++c) {
        const float w = exp2f(base[c * PS + D] - M);
        num = fmaf(base[c * PS + dd], w, num);
        den = fmaf(base[c * PS + D + 1], w, den);
    }
    act_t r;
    from_f32(r, num / den);
    out[(size_t)bv.q_start[s] * Hq * D + h * D + dd] = r;
}

template <int D>
static void launch_decode_d(const act_t* qkv, act_t* out, float* partial, const BatchView& bv, const KvView& kv,
                            int Hq, hipStream_t st) {
    const float scale_log2 = kLog2e / sqrtf((float)D);
    const dim3 grid(bv.decode_chunks, kv.Hkv, bv.n_decode);
    switch (Hq / kv.Hkv) {
        case 1: hipLaunchKernelGGL((attn_decode_kernel<D, 1>), grid, dim3(256), 0, st, qkv, partial, bv, kv, Hq, scale_log2); break;
        case 2: hipLaunchKernelGGL((attn_decode_kernel<D, 2>), grid, dim3(256), 0, st, qkv, partial, bv, kv, Hq, scale_log2); break;
        case 4: hipLaunchKernelGGL((attn_decode_kernel<D, 4>), grid, dim3(256), 0, st, qkv, partial, bv, kv, Hq, scale_log2); break;
        default: hipLaunchKernelGGL((attn_decode_kernel<D, 8>), grid, dim3(256), 0, st, qkv, partial, bv, kv, Hq, scale_log2); break;
    }
    hipLaunchKernelGGL(attn_combine_kernel<D>, dim3(bv.n_decode, Hq), dim3(D), 0, st, partial, out, bv, Hq);
}

void launch_attn_decode(const act_t* qkv, act_t* out, float* partial, const BatchView& bv, const KvView& kv,
                        int Hq, hipStream_t st) {
    if (bv.n_decode <= 0) return;
    if (kv.d == 128) launch_decode_d<128>(qkv, out, partial, bv, kv, Hq, st);
    else launch_decode_d<64>(qkv, out, partial, bv, kv, Hq, st);
}

}  // namespace bz
