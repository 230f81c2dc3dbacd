// Internal definitions shared by the library's host code and kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "blitz_layer.h"

namespace bz {

typedef __bf16 bf16;
typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Activation element: bf16 in the product build, float in the fp32 debug build.
#ifdef BZ_FP32_DEBUG
typedef float act_t;
#else
typedef bf16 act_t;
#endif

constexpr int kWave = 64;

// A kernel's dynamic-LDS limit is a per-function, per-device setting.  One of these per kernel
// instantiation remembers on which devices the limit has been raised (or refused), so that the call is
// made once per device; threads that race here make the same idempotent call.  A refusal is consumed
// here and reported as false, never by a later HIP call.
struct LdsLimit {
    std::atomic<uint64_t> granted{0}, refused{0};
    bool raise(const void* fn, int bytes) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) {
            (void)hipGetLastError();
            return false;
        }
        const uint64_t bit = (dev >= 0 && dev < 64) ? (uint64_t)1 << dev : 0;    // devices past 63: asked every time
        if (granted.load(std::memory_order_acquire) & bit) return true;
        if (refused.load(std::memory_order_acquire) & bit) return false;
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) {
            (void)hipGetLastError();
            refused.fetch_or(bit, std::memory_order_release);
            return false;
        }
        granted.fetch_or(bit, std::memory_order_release);
        return true;
    }
};

// ---- 8-element loads / stores, converting to and from float --------------------------------
__device__ __forceinline__ void load8(const bf16* p, float (&v)[8]) {
    bf16x8 t = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (float)t[i];
}
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
    float4 a = reinterpret_cast<const float4*>(p)[0];
    float4 b = reinterpret_cast<const float4*>(p)[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void store8(bf16* p, const float (&v)[8]) {
    bf16x8 t;
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = (bf16)v[i];
    *reinterpret_cast<bf16x8*>(p) = t;
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
    reinterpret_cast<float4*>(p)[0] = make_float4(v[0], v[1], v[2], v[3]);
    reinterpret_cast<float4*>(p)[1] = make_float4(v[4], v[5], v[6], v[7]);
}
// 8 activation elements kept in their storage format (so loads in flight cost few registers)
struct raw8_bf16 { bf16x8 v; };
struct raw8_f32 { float4 a, b; };
__device__ __forceinline__ void load_raw8(const bf16* p, raw8_bf16& r) { r.v = *reinterpret_cast<const bf16x8*>(p); }
__device__ __forceinline__ void load_raw8(const float* p, raw8_f32& r) {
    r.a = reinterpret_cast<const float4*>(p)[0];
    r.b = reinterpret_cast<const float4*>(p)[1];
}
__device__ __forceinline__ float raw_get(const raw8_bf16& r, int e) { return (float)r.v[e]; }
__device__ __forceinline__ float raw_get(const raw8_f32& r, int e) {
    return e == 0 ? r.a.x : e == 1 ? r.a.y : e == 2 ? r.a.z : e == 3 ? r.a.w
         : e == 4 ? r.b.x : e == 5 ? r.b.y : e == 6 ? r.b.z : r.b.w;
}
#ifdef BZ_FP32_DEBUG
typedef raw8_f32 raw8_act;
#else
typedef raw8_bf16 raw8_act;
#endif

__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ void from_f32(bf16& o, float v) { o = (bf16)v; }
__device__ __forceinline__ void from_f32(float& o, float v) { o = v; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

// Device-side view of the KV cache of one layer.  K part then V part; inside a part, slot s
// starts at element slot_off[s] * Hkv * d and holds Hkv heads of slot_cap[s] positions each
// (slot_cap is a multiple of 32).  Both K and V of one head are stored in blocks of 32 positions,
// each block (32 * d elements, contiguous) in the order in which a 32x32x16 MFMA wants its row
// operand, so attention reads the cache as it lies in memory with 16-byte loads:
//   K (row = position, contraction over d): the 8-element pieces of the head vector are stored
//   piece-major: element (pos, j) lies at k_elem_offset(pos, j, d).  A wave reading piece c of 32
//   consecutive positions touches 512 contiguous bytes.
//   V (row = head dim, contraction over positions): 8 positions form a piece, pieces are stored
//   [piece][j][8].  The 8 positions of piece w = 2t + h are {16t + 4h + 0..3, 16t + 8 + 4h + 0..3}:
//   exactly the positions that lane half h of a 32x32 accumulator holds for k-step t, so softmax
//   probabilities go from the score accumulators into the second MFMA without leaving registers.
__host__ __device__ inline size_t k_piece_offset(int pos, int piece, int d) {
    return (size_t)(pos >> 5) * 32 * d + (((size_t)piece * 32 + (pos & 31)) << 3);
}
__host__ __device__ inline size_t k_elem_offset(int pos, int j, int d) { return k_piece_offset(pos, j >> 3, d) + (j & 7); }
__host__ __device__ inline size_t v_elem_offset(int pos, int j, int d) {
    const int p = pos & 31, t = p >> 4, g = p & 15, h = (g >> 2) & 1, e = (g & 3) + ((g >> 3) << 2);
    return (size_t)(pos >> 5) * 32 * d + (((size_t)(2 * t + h) * d + j) << 3) + e;
}

struct KvView {
    act_t* k;                 // layer's K part
    act_t* v;                 // layer's V part
    const int32_t* slot_off;  // [max_seqs] first token of the slot inside the arena
    const int32_t* slot_cap;  // [max_seqs] capacity in tokens
    int Hkv;
    int d;
};

// Device-side view of a batch.
struct BatchView {
    int B;
    int T;
    const int32_t* q_start;     // [B+1]
    const int32_t* seq_slot;    // [B]
    const int32_t* kv_before;   // [B]
    const int32_t* token_seq;   // [T] sequence index of each packed row
    const int32_t* prefill_items;  // [n_prefill_items][2] = (seq, q_tile)
    int n_prefill_items;
    const int32_t* decode_seqs;    // [n_decode] sequence indices with exactly one new token
    int n_decode;
    int decode_chunks;             // upper bound on ceil((kv_before+1)/kDecodeChunk) over decode seqs
    // One entry (two int4) per (decode sequence, chunk of its cache) that exists now, sequence by
    // sequence: (sequence index, KV slot, index into decode_seqs, chunks of this sequence), (index of
    // the sequence's first entry, 0, 0, 0).  The decode attention runs n_decode_work * Hkv workgroups;
    // workgroup b reads entry b / Hkv, which belongs to the right sequence, and takes
    // (kv head, chunk) = divmod(b - Hkv * first, chunks): a sequence's kv heads one after the other,
    // each head's chunks in order, which is the order the cache lies in memory.
    const int4* decode_work;
    int n_decode_work;
};

constexpr int kPrefillTileQ = 128;   // query rows per prefill-attention workgroup
constexpr int kDecodeChunk = 256;    // KV positions per decode-attention workgroup

// ---- launchers (each enqueues on `st`; shapes are validated by the callers) ------------------
void launch_rmsnorm(const act_t* x, const bf16* gain, act_t* y, int T, int H, float eps, hipStream_t st);
// `ws` is fp32 scratch of at least gemm_workspace_bytes(mode, M, N, K) bytes (0 for shapes that need none);
// without it the decode-sized shapes fall back to a kernel that needs no scratch.
void launch_gemm(int mode, const act_t* a, const bf16* w, const act_t* r, act_t* c, int M, int N, int K,
                 float* ws, size_t ws_bytes, hipStream_t st);
size_t gemm_workspace_bytes(int mode, int M, int N, int K);
// Decode-sized problems only: computes the split-K partial sums partial[ksplit][M][Nrows] (Nrows = 2N
// in SwiGLU mode) into `ws` and returns ksplit, leaving the slice-order reduction and the epilogue
// to the consumer kernel; returns 0 (and does nothing) when the shape does not take that path.
int launch_gemm_partial(int mode, const act_t* a, const bf16* w, int M, int N, int K, float* ws, size_t ws_bytes,
                        hipStream_t st);
// x[T,H] += sum over slices of partial[k][T][H] (slice order), rounded to the activation type and
// stored; then, unless gain is null, y = rmsnorm(x) * gain exactly as launch_rmsnorm would compute it.
void launch_reduce_residual_rmsnorm(act_t* x, const float* partial, int ksplit, const bf16* gain, act_t* y, int T,
                                    int H, float eps, hipStream_t st);
// launch_rope_append on a projection output that is still in split-K partial form
void launch_rope_append_reduce(act_t* qkv, const float* partial, int ksplit, const float* rope_tab,
                               const BatchView& bv, const KvView& kv, int Hq, hipStream_t st);
void launch_rope_append(act_t* qkv, const float* rope_tab, const BatchView& bv, const KvView& kv, int Hq,
                        hipStream_t st);
void launch_attn_prefill(const act_t* qkv, act_t* out, const BatchView& bv, const KvView& kv, int Hq,
                         hipStream_t st);
void launch_attn_decode(const act_t* qkv, act_t* out, float* partial, const BatchView& bv, const KvView& kv,
                        int Hq, hipStream_t st_);
void launch_kv_scatter(const act_t* src_k, const act_t* src_v, const KvView& kv, int slot, int pos0, int n,
                       bool to_cache, act_t* dst_k, act_t* dst_v, hipStream_t st);
// kv_before[s] += 1 for every sequence, then the decode work list is rebuilt for the new lengths
// (at most `capacity` entries are written; the caller has checked that they suffice)
void launch_batch_advance(int32_t* kv_before, int B, const int32_t* decode_seqs, const int32_t* seq_slot, int n_decode,
                          int4* work, int capacity, hipStream_t st);

void launch_set_slot(int32_t* off, int32_t* cap, int32_t off_v, int32_t cap_v, hipStream_t st);

// floats per (decode sequence, query head, chunk) in the decode partial buffer: d outputs, max, sum
__host__ __device__ inline int decode_partial_stride(int d) { return d + 2; }

}  // namespace bz
