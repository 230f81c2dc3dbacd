// HBM-bound steps of a decoder layer: RMSNorm, rotary embedding + KV-cache append, KV scatter /
// gather for cache import/export, and the decode-batch position bump.
#include "common.h"

namespace bz {

// ---------------------------------------------------------------------------------------------
// RMSNorm: one workgroup per token row.  Sum of squares in fp32 (wave shuffle reduction, then a
// fixed-order sum over the waves), y = (x * rstd) * gain rounded once to the activation type.
// ---------------------------------------------------------------------------------------------
// sum over split-K slices, in slice order, of 8 consecutive partial sums of row m.  Loads go out four
// slices at a time (a slice index past the end re-reads the last slice; its value is not added).
__device__ __forceinline__ void reduce8(const float* __restrict__ partial, int ksplit, size_t slice_stride,
                                        size_t off, float (&s)[8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) s[e] = 0.f;
    for (int k0 = 0; k0 < ksplit; k0 += 4) {
        float4 a[4], b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int k = (k0 + u < ksplit) ? k0 + u : ksplit - 1;
            a[u] = *reinterpret_cast<const float4*>(partial + k * slice_stride + off);
            b[u] = *reinterpret_cast<const float4*>(partial + k * slice_stride + off + 4);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (k0 + u < ksplit) {
                s[0] += a[u].x; s[1] += a[u].y; s[2] += a[u].z; s[3] += a[u].w;
                s[4] += b[u].x; s[5] += b[u].y; s[6] += b[u].z; s[7] += b[u].w;
            }
    }
}

// REDUCE: the row of x is first completed as x + (sum of split-K slices), rounded and stored; the
// norm then works on the rounded values, so its result is bit-identical to a separate norm kernel.
// The first kKeep vectors of a thread (rows up to 8 * kKeep * THREADS elements: every supported
// shape) stay in registers between the two passes together with their gains, so the row makes one
// trip from memory.
template <int THREADS, bool REDUCE>
__global__ __launch_bounds__(THREADS) void rmsnorm_kernel(act_t* __restrict__ x, const float* __restrict__ partial,
                                                          int ksplit, int T, const bf16* __restrict__ gain,
                                                          act_t* __restrict__ y, int H, float eps) {
    constexpr int NW = THREADS / kWave;
    constexpr int kKeep = 4;
    __shared__ float red[NW];
    const int row = blockIdx.x;
    act_t* xr = x + (size_t)row * H;
    act_t* yr = y + (size_t)row * H;
    const int nvec = H >> 3;
    float keep[kKeep][8];
    raw8_bf16 gk[kKeep];
    if (gain != nullptr) {
#pragma unroll
        for (int c = 0; c < kKeep; ++c) {
            const int i = threadIdx.x + c * THREADS;
            if (i < nvec) load_raw8(gain + i * 8, gk[c]);
        }
    }
    float ss = 0.f;
    auto first_pass = [&](int i, float (&v)[8]) {
        load8(xr + i * 8, v);
        if (REDUCE) {
            float s[8];
            reduce8(partial, ksplit, (size_t)T * H, (size_t)row * H + i * 8, s);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = s[e] + v[e];
            store8(xr + i * 8, v);
#pragma unroll
            for (int e = 0; e < 8; ++e) {              // continue with the values as stored
                act_t r;
                from_f32(r, v[e]);
                v[e] = to_f32(r);
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = fmaf(v[e], v[e], ss);
    };
#pragma unroll
    for (int c = 0; c < kKeep; ++c) {
        const int i = threadIdx.x + c * THREADS;
        if (i < nvec) first_pass(i, keep[c]);
    }
    for (int i = threadIdx.x + kKeep * THREADS; i < nvec; i += THREADS) {
        float v[8];
        first_pass(i, v);
    }
    if (gain == nullptr) return;
    ss = wave_sum(ss);
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) tot += red[w];
    const float rstd = 1.0f / sqrtf(tot / (float)H + eps);
#pragma unroll
    for (int c = 0; c < kKeep; ++c) {
        const int i = threadIdx.x + c * THREADS;
        if (i < nvec) {
            float o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (keep[c][e] * rstd) * raw_get(gk[c], e);
            store8(yr + i * 8, o);
        }
    }
    for (int i = threadIdx.x + kKeep * THREADS; i < nvec; i += THREADS) {
        float v[8], g[8];
        load8(xr + i * 8, v);
        load8(gain + i * 8, g);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (v[e] * rstd) * g[e];
        store8(yr + i * 8, v);
    }
}

void launch_rmsnorm(const act_t* x, const bf16* gain, act_t* y, int T, int H, float eps, hipStream_t st) {
    if (T <= 0) return;
    act_t* xm = const_cast<act_t*>(x);       // not written without REDUCE
    if (H >= 4096 && T <= 256) {             // few rows: more threads per row shorten each thread's chain of loads
        hipLaunchKernelGGL((rmsnorm_kernel<512, false>), dim3(T), dim3(512), 0, st, xm, nullptr, 0, T, gain, y, H, eps);
    } else if (H >= 2048) {
        hipLaunchKernelGGL((rmsnorm_kernel<256, false>), dim3(T), dim3(256), 0, st, xm, nullptr, 0, T, gain, y, H, eps);
    } else {
        hipLaunchKernelGGL((rmsnorm_kernel<64, false>), dim3(T), dim3(64), 0, st, xm, nullptr, 0, T, gain, y, H, eps);
    }
}

void launch_reduce_residual_rmsnorm(act_t* x, const float* partial, int ksplit, const bf16* gain, act_t* y, int T,
                                    int H, float eps, hipStream_t st) {
    if (T <= 0) return;
    if (H >= 4096 && T <= 256) {
        hipLaunchKernelGGL((rmsnorm_kernel<512, true>), dim3(T), dim3(512), 0, st, x, partial, ksplit, T, gain, y, H, eps);
    } else if (H >= 2048) {
        hipLaunchKernelGGL((rmsnorm_kernel<256, true>), dim3(T), dim3(256), 0, st, x, partial, ksplit, T, gain, y, H, eps);
    } else {
        hipLaunchKernelGGL((rmsnorm_kernel<64, true>), dim3(T), dim3(64), 0, st, x, partial, ksplit, T, gain, y, H, eps);
    }
}

// ---------------------------------------------------------------------------------------------
// Rotary embedding + KV append.  Q is rotated in place inside the packed [T, (Hq+2Hkv)*d]
// projection output; K is rotated and written to the cache; V is copied to the cache.  Pairs are
// (j, j + d/2); the cos/sin table is [max_seq_len][d/2][2] floats built on the host in float64.
//
// Workgroups [n_vblocks, n_vblocks + T) handle one token each (rotation, K write).  The V cache
// keeps 8 positions of one head-dim index in 16 contiguous bytes, so V of a token alone is a
// scatter of single elements: the token's workgroup does that only for positions whose aligned
// group of 16 positions is not written completely by this batch (single-token sequences, ragged
// ends).  Complete groups are written by workgroups [0, n_vblocks): block (prefill item, sub, h)
// gathers the 8 positions of one piece for every (kv head, j) and stores them as one vector.
// ---------------------------------------------------------------------------------------------
template <bool REDUCE>
__global__ __launch_bounds__(256) void rope_append_kernel(act_t* __restrict__ qkv, const float* __restrict__ partial,
                                                          int ksplit, const float* __restrict__ tab, BatchView bv,
                                                          KvView kv, int Hq, int n_vblocks, int tsplit) {
    const int d = kv.d, Hkv = kv.Hkv, half = d >> 1;
    const int nqkv = (Hq + 2 * Hkv) * d;
    if ((int)blockIdx.x < n_vblocks) {
        const int item = blockIdx.x >> 4, sub = (blockIdx.x >> 1) & 7, h = blockIdx.x & 1;
        const int s = bv.prefill_items[2 * item], qt = bv.prefill_items[2 * item + 1];
        const int q0 = bv.q_start[s];
        const int before = bv.kv_before[s];
        const int end = before + (bv.q_start[s + 1] - q0);
        const int grp = ((before + 15) >> 4) + qt * 8 + sub;      // aligned group of 16 positions
        if (grp * 16 + 16 > end) return;
        const int slot = bv.seq_slot[s];
        const int cap = kv.slot_cap[slot];
        const size_t slot_base = (size_t)kv.slot_off[slot] * Hkv * d;
        const int p0 = grp * 16 + 4 * h;                          // the piece holds p0 + {0..3, 8..11}
        const act_t* src = qkv + (size_t)(q0 + (p0 - before)) * nqkv + (size_t)(Hq + Hkv) * d;
        const size_t piece_off = (size_t)(p0 >> 5) * 32 * d + (size_t)(2 * ((p0 >> 4) & 1) + h) * d * 8;
        for (int u = threadIdx.x; u < Hkv * d; u += blockDim.x) {
            const int kvh = u / d, j = u - kvh * d;
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const size_t idx = (size_t)((e & 3) + 8 * (e >> 2)) * nqkv + u;
                if (REDUCE) {
                    const size_t off = (size_t)(src - qkv) + idx;
                    float a = 0.f;
                    for (int k = 0; k < ksplit; ++k) a += partial[k * ((size_t)bv.T * nqkv) + off];
                    act_t r;
                    from_f32(r, a);
                    v[e] = to_f32(r);
                } else {
                    v[e] = to_f32(src[idx]);
                }
            }
            store8(kv.v + slot_base + (size_t)kvh * cap * d + piece_off + (size_t)j * 8, v);
        }
        return;
    }
    // a token's work is shared by `tsplit` workgroups (small batches: more CUs than tokens)
    int t = (blockIdx.x - n_vblocks) / tsplit;
    const int part = (blockIdx.x - n_vblocks) % tsplit;
    if (tsplit == 1) {
        // One workgroup per token: workgroups go to the eight XCDs in turn, and a token's K row is 16-byte
        // pieces that share their 128-byte lines with the 7 neighbouring positions.  Tokens are therefore
        // dealt out in runs of 8 per XCD (n_vblocks is a multiple of 8, so blockIdx.x & 7 is the XCD), and
        // the neighbours' pieces meet in one L2 instead of leaving eight partial lines in eight of them.
        const int xcd = t & 7, seq = t >> 3;
        t = ((seq >> 3) * 8 + xcd) * 8 + (seq & 7);
        if (t >= bv.T) return;
    }
    const int s = bv.token_seq[t];
    const int before = bv.kv_before[s];
    const int pos = before + (t - bv.q_start[s]);
    const int end = before + (bv.q_start[s + 1] - bv.q_start[s]);
    const bool v_by_group = (pos & ~15) >= before && (pos & ~15) + 16 <= end;
    const int slot = bv.seq_slot[s];
    const int cap = kv.slot_cap[slot];
    const size_t slot_base = (size_t)kv.slot_off[slot] * Hkv * d;
    act_t* row = qkv + (size_t)t * nqkv;
    const float* cs = tab + (size_t)pos * d;   // [half][2]
    // REDUCE: the projection output is still split-K partial sums; fold them in slice order and round
    // to the activation type first, exactly as the separate epilogue kernel would have
    auto fetch8 = [&](int col, float (&v)[8]) {
        if (REDUCE) {
            float s8[8];
            reduce8(partial, ksplit, (size_t)bv.T * nqkv, (size_t)t * nqkv + col, s8);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                act_t r;
                from_f32(r, s8[e]);
                v[e] = to_f32(r);
            }
        } else {
            load8(row + col, v);
        }
    };
    const int units_per_head = half >> 3;      // 8 pairs per unit
    const int rot_units = (Hq + Hkv) * units_per_head;
    // V of a token that is stored element by element: first vector requested before the rotation so
    // that both round trips to memory overlap
    constexpr int kPass = 2048;
    const int nv_all = Hkv * d;
    const int v_per = ((nv_all + tsplit - 1) / tsplit + 7) & ~7;          // this workgroup's share of the V row
    const int v_lo = part * v_per;
    const int nv = v_lo >= nv_all ? 0 : (nv_all - v_lo < v_per ? nv_all - v_lo : v_per);
    const int vcol = (Hq + Hkv) * d + v_lo;
    float vpre[8];
    if (!v_by_group && (int)threadIdx.x * 8 < nv) fetch8(vcol + threadIdx.x * 8, vpre);
    for (int u = part * blockDim.x + threadIdx.x; u < rot_units; u += tsplit * blockDim.x) {
        {
            const int head = u / units_per_head;          // 0..Hq-1 query heads, then key heads
            const int j0 = (u - head * units_per_head) * 8;
            act_t* hp = row + head * d;
            float lo[8], hi[8], o_lo[8], o_hi[8];
            fetch8(head * d + j0, lo);
            fetch8(head * d + half + j0, hi);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float c = cs[(j0 + e) * 2], sn = cs[(j0 + e) * 2 + 1];
                o_lo[e] = lo[e] * c - hi[e] * sn;
                o_hi[e] = hi[e] * c + lo[e] * sn;
            }
            if (head < Hq) {
                store8(hp + j0, o_lo);
                store8(hp + half + j0, o_hi);
            } else {
                const int kvh = head - Hq;
                act_t* dst = kv.k + slot_base + (size_t)kvh * cap * d;
                store8(dst + k_piece_offset(pos, j0 >> 3, d), o_lo);
                store8(dst + k_piece_offset(pos, (half + j0) >> 3, d), o_hi);
            }
        }
    }
    if (!v_by_group) {                                  // workgroup-uniform
        // single elements: the row is fetched in vectors and handed over through LDS so that consecutive
        // lanes store consecutive j, i.e. cache addresses 16 bytes apart
        __shared__ act_t vst[kPass];
        for (int base = 0; base < nv; base += kPass) {
            const int cnt = nv - base < kPass ? nv - base : kPass;
            const int u8 = threadIdx.x * 8;
            if (u8 < cnt) {
                if (base > 0) fetch8(vcol + base + u8, vpre);
#pragma unroll
                for (int e = 0; e < 8; ++e) from_f32(vst[u8 + e], vpre[e]);
            }
            __syncthreads();
            for (int u = threadIdx.x; u < cnt; u += blockDim.x) {
                const int kvh = (v_lo + base + u) / d, j = (v_lo + base + u) - kvh * d;
                kv.v[slot_base + (size_t)kvh * cap * d + v_elem_offset(pos, j, d)] = vst[u];
            }
            __syncthreads();
        }
    }
}

void launch_rope_append(act_t* qkv, const float* rope_tab, const BatchView& bv, const KvView& kv, int Hq,
                        hipStream_t st) {
    if (bv.T <= 0) return;
    const int nvb = bv.n_prefill_items * 16;
    const int tsplit = bv.T < 256 ? 4 : 1;
    const int tblocks = tsplit == 1 ? (bv.T + 63) / 64 * 64 : bv.T * tsplit;      // runs of 8 tokens x 8 XCDs
    hipLaunchKernelGGL(rope_append_kernel<false>, dim3(nvb + tblocks), dim3(256), 0, st, qkv, nullptr, 0, rope_tab,
                       bv, kv, Hq, nvb, tsplit);
}

void launch_rope_append_reduce(act_t* qkv, const float* partial, int ksplit, const float* rope_tab,
                               const BatchView& bv, const KvView& kv, int Hq, hipStream_t st) {
    if (bv.T <= 0) return;
    const int nvb = bv.n_prefill_items * 16;
    const int tsplit = bv.T < 256 ? 4 : 1;
    const int tblocks = tsplit == 1 ? (bv.T + 63) / 64 * 64 : bv.T * tsplit;
    hipLaunchKernelGGL(rope_append_kernel<true>, dim3(nvb + tblocks), dim3(256), 0, st, qkv, partial, ksplit,
                       rope_tab, bv, kv, Hq, nvb, tsplit);
}

// ---------------------------------------------------------------------------------------------
// KV scatter/gather between token-major [n, Hkv, d] buffers and the cache layout of one slot.
// K: one thread per 8 head-dim elements of a token (16 bytes on both sides).  V: one thread per
// (piece of 8 positions, kv head, j), 16 bytes on the cache side; pieces that the range
// [pos0, pos0 + n) covers only partly are handled element by element.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void kv_scatter_kernel(const act_t* __restrict__ src_k,
                                                         const act_t* __restrict__ src_v, KvView kv, int slot,
                                                         int pos0, int n, int to_cache,
                                                         act_t* __restrict__ dst_k, act_t* __restrict__ dst_v) {
    const int d = kv.d, Hkv = kv.Hkv;
    const int cap = kv.slot_cap[slot];
    const size_t slot_base = (size_t)kv.slot_off[slot] * Hkv * d;
    const int vec_per_tok = Hkv * (d >> 3);
    const size_t k_total = (size_t)n * vec_per_tok;
    const int piece0 = (pos0 >> 5) * 4;                          // first piece of the first block touched
    const int n_pieces = (((pos0 + n - 1) >> 5) + 1) * 4 - piece0;
    const size_t v_total = (size_t)n_pieces * Hkv * d;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < k_total + v_total;
         i += (size_t)gridDim.x * blockDim.x) {
        if (i < k_total) {
            const int tok = (int)(i / vec_per_tok);
            const int w = (int)(i - (size_t)tok * vec_per_tok);
            const int kvh = w / (d >> 3);
            const int j0 = (w - kvh * (d >> 3)) * 8;
            const size_t lin = (size_t)tok * Hkv * d + (size_t)kvh * d + j0;
            const size_t cac_k = slot_base + (size_t)kvh * cap * d + k_piece_offset(pos0 + tok, j0 >> 3, d);
            float a[8];
            if (to_cache) {
                load8(src_k + lin, a);
                store8(kv.k + cac_k, a);
            } else {
                load8(kv.k + cac_k, a);
                store8(dst_k + lin, a);
            }
        } else {
            const size_t vi = i - k_total;
            const int u = (int)(vi % ((size_t)Hkv * d));          // kvh * d + j: consecutive lanes, consecutive j
            const int piece = piece0 + (int)(vi / ((size_t)Hkv * d));
            const int kvh = u / d, j = u - kvh * d;
            const int w = piece & 3;                              // piece 2t + h of its block
            const int pbase = (piece >> 2) * 32 + 16 * (w >> 1) + 4 * (w & 1);
            act_t* cv = kv.v + slot_base + (size_t)kvh * cap * d + (size_t)(piece >> 2) * 32 * d + ((size_t)w * d + j) * 8;
            const bool whole = pbase >= pos0 && pbase + 11 < pos0 + n;
            if (to_cache) {
                if (whole) {
                    float b[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        b[e] = to_f32(src_v[(size_t)(pbase + (e & 3) + 8 * (e >> 2) - pos0) * Hkv * d + u]);
                    store8(cv, b);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int p = pbase + (e & 3) + 8 * (e >> 2);
                        if (p >= pos0 && p < pos0 + n) cv[e] = src_v[(size_t)(p - pos0) * Hkv * d + u];
                    }
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int p = pbase + (e & 3) + 8 * (e >> 2);
                    if (p >= pos0 && p < pos0 + n) dst_v[(size_t)(p - pos0) * Hkv * d + u] = cv[e];
                }
            }
        }
    }
}

void launch_kv_scatter(const act_t* src_k, const act_t* src_v, const KvView& kv, int slot, int pos0, int n,
                       bool to_cache, act_t* dst_k, act_t* dst_v, hipStream_t st) {
    if (n <= 0) return;
    const size_t n_pieces = (size_t)((((pos0 + n - 1) >> 5) + 1) - (pos0 >> 5)) * 4;
    const size_t total = (size_t)n * kv.Hkv * (kv.d >> 3) + n_pieces * kv.Hkv * kv.d;
    int blocks = (int)((total + 255) / 256);
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(kv_scatter_kernel, dim3(blocks), dim3(256), 0, st, src_k, src_v, kv, slot, pos0, n,
                       to_cache ? 1 : 0, dst_k, dst_v);
}

// One workgroup: moves every sequence one position on, then lists the (sequence, chunk) pairs the decode
// attention has to visit at the new lengths, sequence by sequence (an exclusive scan over chunk counts).
__global__ __launch_bounds__(256) void batch_advance_kernel(int32_t* kv_before, int B, const int32_t* __restrict__ decode_seqs,
                                                            const int32_t* __restrict__ seq_slot, int n_decode, int4* work,
                                                            int capacity) {
    __shared__ int scan[256];
    __shared__ int base;
    const int tid = threadIdx.x;
    for (int i = tid; i < B; i += 256) kv_before[i] += 1;
    if (tid == 0) base = 0;
    __syncthreads();
    for (int d0 = 0; d0 < n_decode; d0 += 256) {
        const int di = d0 + tid;
        int s = 0, n = 0;
        if (di < n_decode) {
            s = decode_seqs[di];
            n = (kv_before[s] + 1 + kDecodeChunk - 1) / kDecodeChunk;
        }
        scan[tid] = n;
        __syncthreads();
        for (int step = 1; step < 256; step <<= 1) {
            const int add = tid >= step ? scan[tid - step] : 0;
            __syncthreads();
            scan[tid] += add;
            __syncthreads();
        }
        const int at = base + scan[tid] - n;
        if (n > 0) {
            const int slot = seq_slot[s];
            for (int c = 0; c < n; ++c)
                if (at + c < capacity) {
                    work[2 * (at + c)] = make_int4(s, slot, di, n);
                    work[2 * (at + c) + 1] = make_int4(at, 0, 0, 0);
                }
        }
        __syncthreads();
        if (tid == 255) base += scan[255];
        __syncthreads();
    }
}

// Slot table entry of one KV slot, written in stream order (a host-to-device copy of four bytes would
// block the calling thread).
__global__ void set_slot_kernel(int32_t* off, int32_t* cap, int32_t off_v, int32_t cap_v) {
    if (threadIdx.x == 0) {
        *off = off_v;
        *cap = cap_v;
    }
}

void launch_set_slot(int32_t* off, int32_t* cap, int32_t off_v, int32_t cap_v, hipStream_t st) {
    hipLaunchKernelGGL(set_slot_kernel, dim3(1), dim3(64), 0, st, off, cap, off_v, cap_v);
}

void launch_batch_advance(int32_t* kv_before, int B, const int32_t* decode_seqs, const int32_t* seq_slot, int n_decode,
                          int4* work, int capacity, hipStream_t st) {
    hipLaunchKernelGGL(batch_advance_kernel, dim3(1), dim3(256), 0, st, kv_before, B, decode_seqs, seq_slot, n_decode, work,
                       capacity);
}

}  // namespace bz
