// gfx950 kernels of the mixed-batch paged-attention path and their launchers.
//
//   kv_append_kernel   scatter this iteration's K/V rows into the paged pools      (HBM-bound)
//   kv_gather_kernel   un-paged copy of one sequence (test hook)                   (HBM-bound)
//   kv_migrate_kernel  pool <-> contiguous transfer buffer, all layers (paper Sec. 3.5)   (HBM-bound)
//   mixed_attention_kernel  ONE launch per layer for the whole mixed batch
//       (paper Sec. 2.2: a prompt chunk plus piggybacked decodes share an iteration):
//         workgroups [0, n_prefill)      causal chunked-prefill pieces: 8 waves = 256 (position, head) rows
//                                        of one KV head over a range of 64-token KV tiles, MFMA 32x32x16,
//                                        software-pipelined so that the softmax runs under the MFMAs
//         remaining workgroups           one decode KV split per wavefront (splits of one sequence and KV head
//                                        that share a workgroup are combined in LDS),
//                                        MFMA 16x16x32 and 16x16x16
//       Two shapes: 8 waves per workgroup, one workgroup per compute unit, when the batch has a prefill
//       chunk; 4 waves, three workgroups per compute unit, for a batch of decodes only.
//       Instantiated for bf16 and IEEE half.
//   split_merge_kernel combine the partial results of split decode sequences and of cut prefill row blocks
//
// Both attention branches compute S^T = K Q^T and O^T = V^T P^T so that the
// probabilities a lane produces are exactly the B operand it must feed to the second
// MFMA (no cross-lane movement), and the per-row softmax state is one scalar per lane.
// The pool layouts (K: [D/8][16][8], V: [D][16] per block and KV head) are the MFMA
// A-operand layouts of those two products, so K/V go from memory to the matrix cores
// without any transposition.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <type_traits>

#include "tc_internal.h"

namespace tc {

typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

// The two 16-bit element types the attention kernels are instantiated for.  Everything that depends
// on the type is here: the vector types, the two MFMA shapes, and (through the casts to `t`) the
// round-to-nearest-even conversions of probabilities and outputs.
struct Bf16 {
    typedef __bf16 t;
    typedef __bf16 x8 __attribute__((ext_vector_type(8)));
    typedef __bf16 x4 __attribute__((ext_vector_type(4)));
    typedef __bf16 x2 __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ f32x16_t mfma32(x8 a, x8 b, f32x16_t c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ f32x4_t mfma16(x8 a, x8 b, f32x4_t c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0); }
    // 16x16x16: contraction over the 16 tokens of one page
    static __device__ __forceinline__ f32x4_t mfma16k16(x4 a, x4 b, f32x4_t c) {
        typedef short s4 __attribute__((ext_vector_type(4)));
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s4, a), __builtin_bit_cast(s4, b), c, 0, 0, 0);
    }
};
struct Fp16 {
    typedef _Float16 t;
    typedef _Float16 x8 __attribute__((ext_vector_type(8)));
    typedef _Float16 x4 __attribute__((ext_vector_type(4)));
    typedef _Float16 x2 __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ f32x16_t mfma32(x8 a, x8 b, f32x16_t c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ f32x4_t mfma16(x8 a, x8 b, f32x4_t c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ f32x4_t mfma16k16(x4 a, x4 b, f32x4_t c) { return __builtin_amdgcn_mfma_f32_16x16x16f16(a, b, c, 0, 0, 0); }
};
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct AttnArgs {
    uint16_t *k_pool, *v_pool;  // written only by the variant that also stores the batch's new rows
    const uint16_t *q;
    const uint16_t *k_new, *v_new;  // this iteration's K/V rows, or null when tc_kv_append has stored them already
    uint16_t *out;
    const int32_t *pages;    // page ids of all sequences, CSR by sequence
    const int32_t *prefill;  // work items
    const int32_t *pieces;   // KV tile ranges of prefill items, stored workgroup by workgroup
    const int32_t *wg_first; // first piece of every prefill workgroup
    const int32_t *decode;
    const int32_t *merge;    // merge items: where the partial results of a split pair lie
    int32_t *counters;       // arrival counters of split pairs; zero before and after every launch
    float *ws_o;             // [n_partials][G][D]
    float *ws_ml;            // [n_partials][G][2]  (running max in the log2 domain, running sum)
    float *ws_pieces;        // piece regions of cut prefill items (PiecePartial), behind the decode partials
    int n_prefill, n_decode; // prefill workgroups, decode wave slots
    int Hq, Hkv, G;
    int fused;               // 1: the last piece or team of a split pair to finish combines its partial results
    int queue;               // index of the decode queue's two counters (next unit, workgroups that have left), or -1
    float scale_log2;        // softmax scale times log2(e)
};

// Position of token `tok` (0..15) inside a 16-token row of the V pool: bits 2 and 3 exchanged, i.e.
// the row holds tokens {0-3, 8-11, 4-7, 12-15}.  Each 16-byte half of a row is then exactly the
// eight contraction slots one half-wave feeds to the 32x32x16 MFMA.  The map is its own inverse.
__host__ __device__ __forceinline__ int v_slot(int tok) { return (tok & 3) | ((tok & 4) << 1) | ((tok & 8) >> 1); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float xor_lanes(float v, int mask) { return __shfl_xor(v, mask, 64); }

// ------------------------------------------------------------------------------------
// KV append / gather
// ------------------------------------------------------------------------------------
// One workgroup writes the rows one sequence adds to one page (1..16 consecutive token indices) for
// one KV head.  K: a thread copies the 16 bytes (8 head-dim elements) of one token.  V is
// token-minor in the pool, so a thread owns one head-dim element and four consecutive token
// slots: it reads up to four 2-byte values (adjacent lanes read adjacent elements, so the reads
// coalesce) and, when all four tokens are new, stores them as one 8-byte word; otherwise it stores
// only the new tokens, 2 bytes each, so every other pool byte stays untouched.
template <int D>
__global__ void __launch_bounds__(4 * D) kv_append_kernel(uint16_t *__restrict__ k_pool, uint16_t *__restrict__ v_pool,
                                                          const uint16_t *__restrict__ k_new,
                                                          const uint16_t *__restrict__ v_new,
                                                          const int32_t *__restrict__ segments, int Hkv) {
    const int32_t *seg = segments + (int64_t)blockIdx.x * kAppendInts;
    const int h = blockIdx.y;
    const int row0 = seg[0], n_tok = seg[1], tok0 = seg[2];
    const int64_t tile = ((int64_t)seg[3] * Hkv + h) * (int64_t)(kBlock * D);
    const int tid = threadIdx.x;
    // ---- V: thread = (slot group g, element d); slots 4g..4g+3 hold tokens t(g)..t(g)+3, t = v_slot(4g)
    {
        const int d = tid % D, g = tid / D;
        const int t_first = v_slot(4 * g);  // token index stored in slot 4g
        uint16_t val[4];
        bool have[4];
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const int t = t_first + e;
            have[e] = t >= tok0 && t < tok0 + n_tok;
            val[e] = have[e] ? v_new[((int64_t)(row0 + t - tok0) * Hkv + h) * D + d] : (uint16_t)0;
        }
        uint16_t *dst = v_pool + tile + (int64_t)d * kBlock + 4 * g;
        if (have[0] && have[1] && have[2] && have[3]) {
            *reinterpret_cast<u32x2 *>(dst) = u32x2{(uint32_t)val[0] | ((uint32_t)val[1] << 16), (uint32_t)val[2] | ((uint32_t)val[3] << 16)};
        } else {
#pragma unroll
            for (int e = 0; e < 4; e++)
                if (have[e]) dst[e] = val[e];
        }
    }
    // ---- K: thread = (token, 8-element piece)
    constexpr int CH = D / 8;
    for (int x = tid; x < n_tok * CH; x += 4 * D) {
        const int i = x / CH, c = x % CH;
        const u32x4 kv = *reinterpret_cast<const u32x4 *>(k_new + ((int64_t)(row0 + i) * Hkv + h) * D + c * 8);
        *reinterpret_cast<u32x4 *>(k_pool + tile + ((int64_t)c * kBlock + tok0 + i) * 8) = kv;
    }
}

template <int D>
__global__ void __launch_bounds__(256) kv_gather_kernel(const uint16_t *__restrict__ k_pool,
                                                        const uint16_t *__restrict__ v_pool,
                                                        const int32_t *__restrict__ pages, int kv_len, int Hkv,
                                                        uint16_t *__restrict__ k_out, uint16_t *__restrict__ v_out) {
    constexpr int CH = D / 8;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)kv_len * Hkv * CH;
    if (gid >= total) return;
    const int c = (int)(gid % CH);
    const int h = (int)((gid / CH) % Hkv);
    const int j = (int)(gid / ((int64_t)CH * Hkv));
    const int64_t blk = pages[j / kBlock];
    const int tok = j % kBlock;
    const int64_t tile = (blk * Hkv + h) * (int64_t)(kBlock * D);
    const int64_t dst = ((int64_t)j * Hkv + h) * D + c * 8;
    *reinterpret_cast<u32x4 *>(k_out + dst) = *reinterpret_cast<const u32x4 *>(k_pool + tile + ((int64_t)c * kBlock + tok) * 8);
    const uint16_t *vsrc = v_pool + tile + (int64_t)(c * 8) * kBlock + v_slot(tok);
    u32x4 vv;
#pragma unroll
    for (int e = 0; e < 4; e++) vv[e] = (uint32_t)vsrc[(2 * e) * kBlock] | ((uint32_t)vsrc[(2 * e + 1) * kBlock] << 16);
    *reinterpret_cast<u32x4 *>(v_out + dst) = vv;
}

// ------------------------------------------------------------------------------------
// KV migration: pool <-> contiguous transfer buffer, every layer in one launch
// ------------------------------------------------------------------------------------
// The transfer buffer is [layers][pages][K block | V block] with both blocks in the pool's own
// layout, so a page moves as 16-byte pieces that are contiguous on both sides; the block id is
// the only indirection.  Workgroup (x, y) moves page x of the selection for layer y.  A full page
// is a straight copy with eight non-temporal loads in flight per thread (the data is touched once).  The last page of a sequence may hold
// fewer than 16 tokens: the export writes zero for the missing ones, the import stores only the
// real ones (K: 16-byte pieces of real tokens; V, which is token-minor: 2-byte elements).
struct MigratePools {
    uint16_t *k[kMigrateLayers];
    uint16_t *v[kMigrateLayers];
};

template <bool IMPORT>
__global__ void __launch_bounds__(256) kv_migrate_kernel(const MigratePools pools, const int32_t *__restrict__ pages,
                                                         const int32_t *__restrict__ valid, uint16_t *__restrict__ buffer,
                                                         int64_t layer_stride, int block_pieces) {
    const int page = blockIdx.x, layer = blockIdx.y;
    const int64_t blk = pages[page];
    const int n_valid = valid[page];
    const int64_t E = (int64_t)block_pieces * 8;  // elements of one block of one pool
    u32x4 *kb = reinterpret_cast<u32x4 *>(buffer + (int64_t)layer * layer_stride + (int64_t)page * 2 * E);
    u32x4 *vb = kb + block_pieces;
    u32x4 *kp = reinterpret_cast<u32x4 *>(pools.k[layer] + blk * E);
    u32x4 *vp = reinterpret_cast<u32x4 *>(pools.v[layer] + blk * E);
    const int tid = threadIdx.x;
    if (n_valid == kBlock) {
        const u32x4 *src_k = IMPORT ? kb : kp, *src_v = IMPORT ? vb : vp;
        u32x4 *dst_k = IMPORT ? kp : kb, *dst_v = IMPORT ? vp : vb;
        constexpr int U = 4;  // pieces of each tensor in flight per thread
        for (int x0 = tid; x0 < block_pieces; x0 += 256 * U) {
            u32x4 a[U], b[U];
#pragma unroll
            for (int u = 0; u < U; u++) {
                const int x = x0 + 256 * u;
                if (x < block_pieces) {
                    a[u] = __builtin_nontemporal_load(src_k + x);
                    b[u] = __builtin_nontemporal_load(src_v + x);
                }
            }
#pragma unroll
            for (int u = 0; u < U; u++) {
                const int x = x0 + 256 * u;
                if (x < block_pieces) {
                    __builtin_nontemporal_store(a[u], dst_k + x);
                    __builtin_nontemporal_store(b[u], dst_v + x);
                }
            }
        }
        return;
    }
    for (int x = tid; x < block_pieces; x += 256) {
        // K piece x = (head, d/8, token): the token index is the piece index mod 16
        const bool real = (x & (kBlock - 1)) < n_valid;
        if (IMPORT) {
            if (real) kp[x] = kb[x];
        } else {
            kb[x] = real ? kp[x] : u32x4{0u, 0u, 0u, 0u};
        }
        // V piece x = (head, d, half row): slots 8*(x&1) .. +7, slot s holds token v_slot(s)
        const int slot0 = (x & 1) * 8;
        if (IMPORT) {
            const u32x4 w = vb[x];
            uint16_t *dst = reinterpret_cast<uint16_t *>(vp + x);
#pragma unroll
            for (int e = 0; e < 8; e++)
                if (v_slot(slot0 + e) < n_valid) dst[e] = (uint16_t)(w[e >> 1] >> ((e & 1) * 16));
        } else {
            u32x4 w = vp[x];
#pragma unroll
            for (int e = 0; e < 8; e++)
                if (v_slot(slot0 + e) >= n_valid) w[e >> 1] &= (e & 1) ? 0x0000FFFFu : 0xFFFF0000u;
            vb[x] = w;
        }
    }
}

// ------------------------------------------------------------------------------------
// Combination of partial results
// ------------------------------------------------------------------------------------
// Partial results that are combined inside the attention kernel cross from one compute unit to another
// (possibly on another die, with an L2 cache of its own) while the kernel runs.  They are written and read
// with device-scope atomic stores and loads (relaxed; 8 bytes each; the large piece regions with 16-byte
// accesses that carry the same cache policy, see peer_window), which go past the caches that are not
// coherent across the device, so no cache has to be written back or invalidated as a whole: a release
// and an acquire fence per piece (an L2 write-back and an L2 invalidate, by every wave) measured twice
// the kernel time on a levelled 2048-token chunk.  Ordering is by the arrival counter: a writer waits
// until its stores have completed (s_waitcnt) before it counts itself in; the reader is the part that sees
// the full count.  PEER = false: the plain loads of the merge launch, which runs after the kernel has ended.
__device__ __forceinline__ void peer_store2(float *p, float a, float b) {
    const uint64_t bits = (uint64_t)__float_as_uint(a) | ((uint64_t)__float_as_uint(b) << 32);
    __hip_atomic_store(reinterpret_cast<uint64_t *>(p), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <bool PEER>
__device__ __forceinline__ float2 load2(const float *p) {
    if (!PEER) return *reinterpret_cast<const float2 *>(p);
    const uint64_t bits = __hip_atomic_load(reinterpret_cast<const uint64_t *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return float2{__uint_as_float((uint32_t)bits), __uint_as_float((uint32_t)(bits >> 32))};
}
template <bool PEER>
__device__ __forceinline__ float load1(const float *p) {
    if (!PEER) return *p;
    return __uint_as_float(__hip_atomic_load(reinterpret_cast<const uint32_t *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// 16 bytes at a time, for the piece regions (133 KiB each): buffer loads and stores that carry the cache policy of
// a device-scope atomic access (the sc1 bit; the access goes past the caches that are not coherent across the
// device) without being atomic, which no 16-byte access can be.  Nothing needs them to be: a region is complete
// before its arrival is counted, and is read only after the count is full.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
constexpr int kCoherentAux = 16;  // sc1
__device__ __forceinline__ __amdgpu_buffer_rsrc_t peer_window(const float *base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(base), 0, (int)bytes, 0x00020000);  // raw dwords, no stride
}
template <bool PEER>
__device__ __forceinline__ f32x4 load4(__amdgpu_buffer_rsrc_t win, const float *base, uint32_t byte_off) {
    if (!PEER) return *reinterpret_cast<const f32x4 *>(reinterpret_cast<const char *>(base) + byte_off);
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(win, (int)byte_off, 0, kCoherentAux));
}
__device__ __forceinline__ void peer_store4(__amdgpu_buffer_rsrc_t win, uint32_t byte_off, f32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, v), win, (int)byte_off, 0, kCoherentAux);
}

// One output row (query head j of a decode sequence, or of one position of a cut prefill item) from its
// ns partial results in workspace slots slot0 .. slot0 + ns - 1:
//   out = sum_i 2^(m_i - m*) o_i / sum_i 2^(m_i - m*) l_i,   m* = max_i m_i,   partials in index order.
// One wavefront per row; a lane owns D/64 adjacent head-dim elements, so each partial row is one coalesced
// read.  Lane i first fetches (m_i, l_i) of partial i (at most 64 per pass; passes are chained by an online
// rescale), the wave reduces the maximum, and the weighted sum runs over the partials in index order with
// the weights broadcast from those registers.  The order is fixed, so the result does not depend on which
// workgroup runs this or when.
template <int D, class E, bool PEER>
__device__ __forceinline__ void merge_row(const float *ws_o, const float *ws_ml, int64_t slot0, int ns, int G, int j,
                                          uint16_t *dst_row, int lane) {
    constexpr int NE = D / 64;  // elements per lane
    float acc[NE];
#pragma unroll
    for (int e = 0; e < NE; e++) acc[e] = 0.f;
    float m_star = -1e30f, den = 0.f;
    for (int base = 0; base < ns; base += 64) {
        const int n = min(64, ns - base);
        const float *src = ws_o + ((int64_t)(slot0 + base) * G + j) * D + lane * NE;
        // Partial rows are fetched kChunk at a time, all loads of a chunk in flight together; the
        // first chunk is requested before the weights are known.
        constexpr int kChunk = 8;
        float row[kChunk][NE];
        auto fetch = [&](int c0) {
#pragma unroll
            for (int u = 0; u < kChunk; u++)
                if (c0 + u < n) {
                    const float *r = src + (int64_t)(c0 + u) * G * D;
                    if (NE == 2) {
                        const float2 v = load2<PEER>(r);
                        row[u][0] = v.x;
                        row[u][NE - 1] = v.y;
                    } else {
                        row[u][0] = load1<PEER>(r);
                    }
                }
        };
        fetch(0);
        const int64_t my_row = (int64_t)(slot0 + base + min(lane, n - 1)) * G + j;
        const float2 ml = load2<PEER>(ws_ml + my_row * 2);  // lanes past n read the last partial's pair and ignore it
        const float m_i = lane < n ? ml.x : -1e30f;
        const float l_i = lane < n ? ml.y : 0.f;
        float m_new = m_i;
#pragma unroll
        for (int sh = 1; sh < 64; sh *= 2) m_new = fmaxf(m_new, xor_lanes(m_new, sh));
        m_new = fmaxf(m_new, m_star);
        const float rescale = fast_exp2(m_star - m_new);
        m_star = m_new;
        const float w_i = fast_exp2(m_i - m_star);  // 0 for lanes past n
        float wl = w_i * l_i;
#pragma unroll
        for (int sh = 1; sh < 64; sh *= 2) wl += xor_lanes(wl, sh);
        den = den * rescale + wl;
#pragma unroll
        for (int e = 0; e < NE; e++) acc[e] *= rescale;
        for (int c0 = 0; c0 < n; c0 += kChunk) {
#pragma unroll
            for (int u = 0; u < kChunk; u++)
                if (c0 + u < n) {
                    const float w = __shfl(w_i, c0 + u, 64);
#pragma unroll
                    for (int e = 0; e < NE; e++) acc[e] += w * row[u][e];
                }
            if (c0 + kChunk < n) fetch(c0 + kChunk);
        }
    }
    const float inv = 1.f / den;
    uint16_t *dst = dst_row + lane * NE;
    if (NE == 2) {
        typename E::x2 w2;
        w2[0] = (typename E::t)(acc[0] * inv);
        w2[1] = (typename E::t)(acc[NE - 1] * inv);
        *reinterpret_cast<typename E::x2 *>(dst) = w2;
    } else {
        const typename E::t w1 = (typename E::t)(acc[0] * inv);
        *dst = __builtin_bit_cast(uint16_t, w1);
    }
}

// Arrival of one of the n parts of a split pair, after the part has stored its partial result with
// peer_store2 and the stores have completed: the pair's counter is incremented.  Returns true to the part
// that arrives last; that part combines the partial results (reading them with PEER loads) and puts the
// counter back to zero for the next launch.  Nobody waits for anybody.
// `leader`: the one lane that does the counting; all lanes of the calling wave get its answer.
__device__ __forceinline__ bool arrive_is_last(int32_t *counter, int n, bool leader) {
    stores_done();
    int old = 0;
    if (leader) old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __builtin_amdgcn_readfirstlane(old);
    return old == n - 1;
}

// Partial result of one piece of a cut prefill item: what the 512 lanes of the workgroup hold at the end of
// the piece's sweep, stored as it lies in registers.  Lane (wave, n = lane % 32, hh = lane / 32) owns row
// wave * 32 + n and, of its D accumulators, those at head-dim positions 32 c + 8 q + 4 hh .. + 3 (c < D/32, q < 4).
//   o:  [wave][chunk = 4 c + q][lane][4] floats   one store instruction of a wave = 1 KiB contiguous
//   ml: [wave][n][2] floats                         (running maximum in the log2 domain, row sum)
// The combination reads the K partial results of an item back in the same layout, so it needs no exchange
// between lanes and all its loads are independent:
//   o = sum_i 2^(m_i - m*) o_i,  l = sum_i 2^(m_i - m*) l_i,  m* = max_i m_i,  pieces in index order,
// which leaves the lane with the accumulators and row sum of the whole item, as after an uncut sweep.
template <int D>
struct PiecePartial {
    static constexpr int MT = D / 32;
    static constexpr int kChunks = 4 * MT;
    static constexpr int kOFloats = kMixedWaves * kChunks * 64 * 4;  // = kPrefillRows * D
    static constexpr int kFloats = kOFloats + kPrefillRows * 2;
    static constexpr uint32_t kBytes = (uint32_t)kFloats * sizeof(float);
    static __device__ __forceinline__ uint32_t lane_offset(int wave, int lane) { return (uint32_t)((wave * kChunks * 64 + lane) * 4 * sizeof(float)); }
    static __device__ __forceinline__ void store(float *region, int wave, int lane, const f32x16 (&o)[MT], float m, float l, bool peer) {
        float *dst = region + ((int64_t)wave * kChunks * 64 + lane) * 4;
        float *ml = region + kOFloats + (wave * 32 + (lane & 31)) * 2;
        if (peer) {
            const __amdgpu_buffer_rsrc_t win = peer_window(region, kBytes);
            const uint32_t at = lane_offset(wave, lane);
#pragma unroll
            for (int c = 0; c < MT; c++)
#pragma unroll
                for (int q = 0; q < 4; q++)
                    peer_store4(win, at + (4 * c + q) * 1024, f32x4{o[c][4 * q], o[c][4 * q + 1], o[c][4 * q + 2], o[c][4 * q + 3]});
            if (lane < 32) peer_store2(ml, m, l);
        } else {
#pragma unroll
            for (int c = 0; c < MT; c++)
#pragma unroll
                for (int q = 0; q < 4; q++)
                    __builtin_nontemporal_store(f32x4{o[c][4 * q], o[c][4 * q + 1], o[c][4 * q + 2], o[c][4 * q + 3]},
                                                reinterpret_cast<f32x4 *>(dst + (4 * c + q) * 256));
            if (lane < 32) {
                ml[0] = m;
                ml[1] = l;
            }
        }
    }
    // `first`: region of the item's piece 0; the K regions follow each other.  The accumulators of piece i + 1 are
    // requested before those of piece i are added, so that a piece's worth of loads is always in flight.
    template <bool PEER>
    static __device__ __forceinline__ void combine(const float *first, int k, int wave, int lane, f32x16 (&o)[MT], float &l) {
        const float *ml = first + kOFloats + (wave * 32 + (lane & 31)) * 2;
        const __amdgpu_buffer_rsrc_t win = peer_window(first, (uint32_t)k * kBytes);
        const uint32_t at = lane_offset(wave, lane);
        auto fetch = [&](int i, f32x4 (&t)[kChunks], float2 &mli) {
            mli = load2<PEER>(ml + (int64_t)i * kFloats);
#pragma unroll
            for (int ch = 0; ch < kChunks; ch++) t[ch] = load4<PEER>(win, first, (uint32_t)i * kBytes + at + ch * 1024);
        };
        f32x4 t_cur[kChunks], t_nxt[kChunks];
        float2 ml_cur, ml_nxt;
        fetch(0, t_cur, ml_cur);
        float m_star = -1e30f;
        for (int i = 0; i < k; i++) m_star = fmaxf(m_star, load2<PEER>(ml + (int64_t)i * kFloats).x);
#pragma unroll
        for (int c = 0; c < MT; c++)
#pragma unroll
            for (int r = 0; r < 16; r++) o[c][r] = 0.f;
        l = 0.f;
        for (int i = 0; i < k; i++) {
            if (i + 1 < k) fetch(i + 1, t_nxt, ml_nxt);
            const float w = fast_exp2(ml_cur.x - m_star);
            l += w * ml_cur.y;
#pragma unroll
            for (int c = 0; c < MT; c++)
#pragma unroll
                for (int r = 0; r < 16; r++) o[c][r] += w * t_cur[4 * c + (r >> 2)][r & 3];
#pragma unroll
            for (int ch = 0; ch < kChunks; ch++) t_cur[ch] = t_nxt[ch];
            ml_cur = ml_nxt;
        }
    }
};

// Output rows of a prefill item from a lane's accumulators and its row's sum: o / l, rounded to the element type.
template <int D, class E>
__device__ __forceinline__ void prefill_write_rows(uint16_t *row, const f32x16 (&o)[D / 32], float l, int hh) {
    typedef typename E::x4 x4;
    typedef typename E::t el;
    const float inv = 1.f / l;
#pragma unroll
    for (int c = 0; c < D / 32; c++)
#pragma unroll
        for (int q4 = 0; q4 < 4; q4++) {
            x4 w;
#pragma unroll
            for (int e = 0; e < 4; e++) w[e] = (el)(o[c][4 * q4 + e] * inv);
            *reinterpret_cast<x4 *>(row + 32 * c + 8 * q4 + 4 * hh) = w;
        }
}

// ------------------------------------------------------------------------------------
// Prefill branch: one workgroup = 256 (position, head) rows of one KV head, 32 per wave.
// ------------------------------------------------------------------------------------
// Row R of the workgroup is position first_pos + R / G, query head kv_head * G + R % G.
// The KV range 0..last position is swept in 64-token tiles (four pages); each tile is
// copied page by page into LDS exactly as it lies in the pool and consumed by
//   S^T[token][row]  = sum_d K[token][d] Q[row][d]        (A = K from LDS, B = Q in registers)
//   O^T[d][row]     += sum_token V^T[d][token] P^T[token][row]   (A = V^T from LDS, B = P)
// with the online softmax (running max m, running sum l) kept per row in fp32.

template <int D>
struct PrefillCfg {
    static constexpr int kTileTokens = 64;
    static constexpr int kTilePages = kTileTokens / kBlock;
    static constexpr int kPageBytes = kBlock * D * 2;               // one (page, KV head) tile of K or of V
    static constexpr int kTileBytes = kTilePages * kPageBytes;      // K part or V part of one LDS stage
    static constexpr int kRuns = kPageBytes / 1024;                 // 1 KiB wave-wide loads per page and tensor
    // kStages LDS stages of K and of V: a tile is copied kStages - 1 steps before its first use.
    // 96 KiB at D = 128.  (A fourth stage, 128 KiB, measured no faster; the pipeline below is written in
    // terms of kStages, but three is the only depth that is built and tested.)
    static constexpr int kStages = 3;
    static_assert(kStages == 3, "three stages is the only depth that is built and tested");
    static constexpr int kIdSlots = kStages - 2;  // page ids in flight per copying wave and tensor
    static constexpr int kQueueSlot = 2 * kStages * kTileBytes + kMixedWaves * kIdSlots * 64 * 4;  // where a workgroup keeps the decode unit it drew
    static constexpr int kLdsBytes = kQueueSlot + 16;
};

// N direct-to-LDS loads of 1 KiB each (16 bytes per lane) at immediate offsets 0, 1024, ...
template <int N>
__device__ __forceinline__ void lds_load_runs(const __attribute__((address_space(1))) void *src,
                                              __attribute__((address_space(3))) void *dst) {
    static_assert(N >= 1 && N <= 4, "the immediate offset field holds up to 4095");
    __builtin_amdgcn_global_load_lds(src, dst, 16, 0, 0);
    if constexpr (N > 1) __builtin_amdgcn_global_load_lds(src, dst, 16, 1024, 0);
    if constexpr (N > 2) __builtin_amdgcn_global_load_lds(src, dst, 16, 2048, 0);
    if constexpr (N > 3) __builtin_amdgcn_global_load_lds(src, dst, 16, 3072, 0);
}

// Page id of page `page_in_tile` of KV tile `tile` (a scalar load; past the end of the sequence the
// last page is named, whose copy is never used).
template <int D>
__device__ __forceinline__ int prefill_page_id(const int32_t *__restrict__ pages, int n_pages, int tile, int page_in_tile) {
    return pages[min(tile * PrefillCfg<D>::kTilePages + page_in_tile, n_pages - 1)];
}

// Tile copies.  The 8 waves of a workgroup share every tile.  A copier moves one page of a tile (copier
// index 0-3: the four K pages, 4-7: the four V^T pages) with direct-to-LDS loads: lane L deposits its 16 bytes at
// (wave-uniform base) + 16 L, so each load copies a 1 KiB run; the runs of a page are contiguous both
// in the pool and in LDS, so they share one address register and one LDS base and differ only in the
// instruction's immediate offset.  K pages are copied verbatim.  A V^T page is copied row by row
// (32 bytes = 16 token slots of one head-dim element) with the two 16-byte halves of rows 8-15
// (mod 16) exchanged, so that the operand reads of 16 consecutive rows cover all 64 LDS banks (a
// 1 KiB step is 32 rows, so the exchange pattern is the same in every run).
template <int D>
struct TileCopier {
    using C = PrefillCfg<D>;
    typedef const __attribute__((address_space(1))) void *gptr_t;
    typedef __attribute__((address_space(3))) void *lptr_t;
    const uint16_t *src;  // pool + this lane's element offset inside a (page, KV head) block
    char *dst;            // stage 0 of this wave's tensor + its page slot
    int64_t head_off;     // kv head * block elements
    int64_t page_stride;  // elements per page (all KV heads)
    bool is_v;
    int page_in_tile;
    __device__ __forceinline__ TileCopier(const AttnArgs &A, int kvh, char *lds_k, char *lds_v, int wave, int lane) {  // wave = copier index
        static_assert(2 * C::kTilePages == kMixedWaves, "the waves 0 .. kTilePages - 1 are the older wave of each SIMD");
        static_assert(C::kTileTokens == kPrefillTileTokens, "the planner cuts KV ranges in units of this tile");
        is_v = wave >= C::kTilePages;
        page_in_tile = wave & (C::kTilePages - 1);
        const int d = lane >> 1, half = (lane & 1) ^ ((d >> 3) & 1);
        src = is_v ? A.v_pool + d * kBlock + half * 8 : A.k_pool + lane * 8;
        dst = (is_v ? lds_v : lds_k) + page_in_tile * C::kPageBytes;
        head_off = (int64_t)kvh * (kBlock * D);
        page_stride = (int64_t)A.Hkv * (kBlock * D);
    }
    // copy this wave's page (wave-uniform id) into LDS stage `stage` of its tensor
    __device__ __forceinline__ void copy(int page_id, int stage) const {
        const int64_t base = (int64_t)__builtin_amdgcn_readfirstlane(page_id) * page_stride + head_off;
        lds_load_runs<C::kRuns>((gptr_t)(src + base), (lptr_t)(dst + stage * C::kTileBytes));
    }
};

// After this thread's own direct-to-LDS loads of `tile` have landed: slots at or past `kv_len`
// hold undefined bits (the tail of the last page, or a clamped re-read of it for pages past the
// end).  They get probability 0 but must be finite for the MFMA, so zero them in the V stage.
// Each thread patches only the 16-byte pieces it loaded itself (`wave` = the page of the tile this
// wave copied), so no extra barrier is needed.
template <int D>
__device__ __forceinline__ void prefill_fix_tail(char *lds_v, int tile, int wave, int lane, int kv_len) {
    using C = PrefillCfg<D>;
    const int n_valid = kv_len - (tile * C::kTilePages + wave) * kBlock;
    if (n_valid < kBlock) {
        const int d = lane >> 1, half = (lane & 1) ^ ((d >> 3) & 1);
#pragma unroll
        for (int i = 0; i < C::kRuns; i++) {
            u32x4 *piece = reinterpret_cast<u32x4 *>(lds_v + wave * C::kPageBytes + i * 1024 + lane * 16);
            u32x4 vv = *piece;
#pragma unroll
            for (int e = 0; e < 4; e++) {
                uint32_t w = vv[e];
                if (v_slot(half * 8 + 2 * e) >= n_valid) w &= 0xFFFF0000u;
                if (v_slot(half * 8 + 2 * e + 1) >= n_valid) w &= 0x0000FFFFu;
                vv[e] = w;
            }
            *piece = vv;
        }
    }
}

__device__ __forceinline__ void wait_all_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// The page id of a wave's future tile copy is fetched with a direct-to-LDS load into a slot of the
// wave's own (every lane loads the same id and deposits it at slot + 4 * lane): it is counted by
// vmcnt like the tile copies (a scalar load in flight would force the LDS operand reads to wait
// for everything), and no register is ever pending: the value is read from LDS after the wait.
constexpr int kIdSlotBytes = 64 * 4;
__device__ __forceinline__ void page_id_fetch(const int32_t *p, char *slot) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)p, (__attribute__((address_space(3))) void *)slot, 4, 0, 0);
}
template <int N>  // wait until at most the N most recent loads of this wave are in flight
__device__ __forceinline__ void wait_loads_but() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
__device__ __forceinline__ int page_id_read(const char *slot, int lane) {
    return __builtin_amdgcn_readfirstlane(*reinterpret_cast<const int *>(slot + 4 * lane));
}

// max / sum across the two half-waves (lanes l and l ^ 32 hold the two halves of a row).
__device__ __forceinline__ float half_swap_max(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_swap_sum(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// One wave's share of the two products and of the softmax, for 32 rows x 32 tokens (half a tile).
template <int D, class E>
struct PrefillWave {
    using C = PrefillCfg<D>;
    using x8 = typename E::x8;
    using el = typename E::t;
    static constexpr int KS = D / 16;  // k-steps of the QK^T product
    static constexpr int MT = D / 32;  // 32-row tiles of O^T

    // K fragments (MFMA A operands) of tokens 32 h .. 32 h + 31 of a K stage; kp = stage base + lane offset.
    typedef const __attribute__((address_space(3))) char *lds_cptr;
    typedef const __attribute__((address_space(3))) x8 *lds_x8ptr;
    static __device__ __forceinline__ void load_k(lds_cptr kp, int h, x8 (&kf)[KS]) {
#pragma unroll
        for (int kk = 0; kk < KS; kk++) kf[kk] = *(lds_x8ptr)(kp + 2 * h * C::kPageBytes + 2 * kk * (kBlock * 16));
    }
    // V^T fragments of the two pages of half h of a V stage; vp = stage base + lane offset.
    static __device__ __forceinline__ void load_v(lds_cptr vp, int h, x8 (&vf)[2][MT]) {
#pragma unroll
        for (int b = 0; b < 2; b++)
#pragma unroll
            for (int c = 0; c < MT; c++) vf[b][c] = *(lds_x8ptr)(vp + (2 * h + b) * C::kPageBytes + c * (32 * 32));
    }
    // S^T = K Q^T for 32 tokens
    static __device__ __forceinline__ void qk(const x8 (&kf)[KS], const x8 (&qreg)[KS], f32x16 &s) {
#pragma unroll
        for (int r = 0; r < 16; r++) s[r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KS; kk++) s = E::mfma32(kf[kk], qreg[kk], s);
    }
    // Scores of tokens past the row's own position become -inf (probability 0); tok0 = first token of the half.
    static __device__ __forceinline__ void causal_mask(f32x16 &s, int tok0, int hh, int p_abs) {
#pragma unroll
        for (int r = 0; r < 16; r++) {
            const int j = tok0 + 8 * (r >> 2) + 4 * hh + (r & 3);
            s[r] = (j <= p_abs) ? s[r] : -INFINITY;
        }
    }
    // Row maximum over the 32 tokens (both half-waves).
    static __device__ __forceinline__ float row_max(const f32x16 &s) {
        float mx = s[0];
#pragma unroll
        for (int r = 1; r < 16; r++) mx = fmaxf(mx, s[r]);
        return half_swap_max(mx);
    }
    // p = 2^(s * c - m), rounded to the element type as the B operand of the second product (one
    // operand per page); psum = this lane's sum of the unrounded values.  (Summing the rounded pairs with
    // one dot-product instruction per pair measured 9 % slower.)
    static __device__ __forceinline__ void probs(const f32x16 &s, float c_log2, float m_run, x8 (&pb)[2], float &psum) {
        psum = 0.f;
#pragma unroll
        for (int b = 0; b < 2; b++)
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const float pv = fast_exp2(__builtin_fmaf(s[8 * b + e], c_log2, -m_run));
                psum += pv;
                pb[b][e] = (el)pv;
            }
    }
    // O^T += V^T P^T over 32 tokens
    static __device__ __forceinline__ void pv(const x8 (&vf)[2][MT], const x8 (&pb)[2], f32x16 (&o)[MT]) {
#pragma unroll
        for (int b = 0; b < 2; b++)
#pragma unroll
            for (int c = 0; c < MT; c++) o[c] = E::mfma32(vf[b][c], pb[b], o[c]);
    }
};

// The reference maximum of a row (log2 domain) is kept while it serves: probabilities may exceed 1 as long
// as fp32 sums and 16-bit operands hold them without loss of relative precision, so O has to be rescaled
// only a few times per sweep instead of whenever any of a wave's 32 rows sees a new maximum, and the row
// maxima themselves need not be computed per tile.  The probabilities of a half-tile are computed with
// the reference as it is; if a lane's sum of them exceeds kSumLimit (some probability is above 2^9), the
// wave computes the true row maxima of that half-tile, moves the reference of every row whose maximum
// exceeds it by more than kMaxSlack, and computes the probabilities again (`settle` in prefill_item).
constexpr float kMaxSlack = 8.f;
constexpr float kSumLimit = 8192.f;  // 16 probabilities of at most 2^9
__device__ __forceinline__ float next_reference_max(float m_run, float row_max_log2) {
    return row_max_log2 > m_run + kMaxSlack ? row_max_log2 : m_run;
}

// The KV sweep is software-pipelined inside every wave, in units of half a tile (32 tokens), three
// halves deep: in one phase the matrix cores compute the scores of half h + 1 and accumulate P V of
// half h - 1 while the vector ALU turns the scores of half h into probabilities.  (MFMA and VALU
// instructions of one wave overlap fully when they are interleaved in the instruction stream;
// executed one after the other their times add up.)  The LDS read that refills an MFMA's operand
// register for the next phase follows that MFMA, a whole phase ahead of its use.  The 8 waves share
// the K/V tiles; a tile is copied two steps ahead of its first use, so one barrier per tile suffices
// and no wave waits for a copy:
//   step j:  barrier | waves 0-3: copy K(j+3) and V(j+2) | phase 2j | phase 2j + 1
//            | waves 0-3: wait for the copies issued in step j - 1
// Waves 0-3 are the older wave of their SIMDs: the hardware issues their instructions first, they finish
// a step's phases early and would wait at the barrier, so the copies cost them nothing, while waves 4-7,
// which set the pace, are spared them (1 % on a long sweep; copies by waves 4-7 alone measured 0.2 %
// slower than one tensor per wave group).
template <int D, class E>
__device__ void prefill_item(const AttnArgs &A, const int32_t *__restrict__ it, const int32_t *__restrict__ pc, char *lds) {
    using C = PrefillCfg<D>;
    using W = PrefillWave<D, E>;
    using x8 = typename E::x8;
    using el = typename E::t;
    typedef typename W::lds_cptr lds_cptr;
    constexpr int KS = W::KS, MT = W::MT;
    // A workgroup may run several pieces in a loop.  Everything a lane derives from its index is derived again
    // for every piece (the empty asm hides that the index does not change): hoisted out of that loop, the
    // values only the start of a piece needs would occupy registers throughout the sweep, which has none to spare.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, hh = lane >> 5;
    const int kvh = it[PF_KVH], pos0 = it[PF_POS0], npos = it[PF_NPOS], qrow0 = it[PF_QROW0], ctx = it[PF_CTX];
    const int n_pages = it[PF_NPAGES];
    const int32_t *pages = A.pages + it[PF_PAGEOFF];
    const int G = A.G;
    const int n_rows = npos * G;
    // this lane's row of the workgroup's 256: position pos0 + R / G, head kvh * G + R % G
    const int R = wave * 32 + n;
    const bool row_valid = R < n_rows;
    const int Rc = row_valid ? R : n_rows - 1;
    const int p_abs = ctx + pos0 + Rc / G;  // the row attends over tokens 0..p_abs
    const int64_t row_off = ((int64_t)(qrow0 + pos0 + Rc / G) * A.Hq + kvh * G + Rc % G) * D;
    // first position of the rows this wave owns (wave-uniform): tiles that end at or before it need no mask
    const int wave_pmin = ctx + pos0 + min(wave * 32, n_rows - 1) / G;
    const int kv_len = ctx + pos0 + npos;  // tokens this workgroup may read (all appended already)
    // KV tiles [t_begin, t_end) of the item; p_slot < 0: the whole range, results go to `out`
    const int t_begin = pc[PP_T0], t_end = pc[PP_T1], p_slot = pc[PP_SLOT], p_k = pc[PP_K];
    const int n_sweep = t_end - t_begin;
    const float c_log2 = A.scale_log2;
    char *const lds_k = lds, *const lds_v = lds + C::kStages * C::kTileBytes;
    // per-lane byte offsets of the MFMA A operands inside a stage
    const int k_lane_off = (n >> 4) * C::kPageBytes + (n & 15) * 16 + hh * (kBlock * 16);
    const int v_lane_off = n * 32 + ((hh ^ ((n >> 3) & 1)) * 16);

    x8 qreg[KS];
#pragma unroll
    for (int kk = 0; kk < KS; kk++) qreg[kk] = *reinterpret_cast<const x8 *>(A.q + row_off + (2 * kk + hh) * 8);

    f32x16 o[MT];
#pragma unroll
    for (int c = 0; c < MT; c++)
#pragma unroll
        for (int r = 0; r < 16; r++) o[c][r] = 0.f;
    float m_run = -1e30f;  // running row maximum (log2 domain)
    float l_run = 0.f;     // running sum of this lane's half of the row

    // ---- prologue: tile j of the sweep lives in stage j mod NS of its tensor.  K(0..NS-1) and V(0..NS-2)
    // are copied here; step j then copies K(j+NS) and V(j+NS-1).
    constexpr int NS = C::kStages;
    // Waves 0-3 copy both tensors: wave w page w of the K tile and of the V tile.  Waves 4-7 issue no loads.
    const bool copier = wave < C::kTilePages;
    const TileCopier<D> cpk(A, kvh, lds_k, lds_v, wave & (C::kTilePages - 1), lane);
    const TileCopier<D> cpv(A, kvh, lds_k, lds_v, (wave & (C::kTilePages - 1)) + C::kTilePages, lane);
    const int pg = cpk.page_in_tile;
    int idk_cur = 0, idv_cur = 0;  // pages this wave copies in step 0
    // The page ids for the copies of step j are fetched in step j - (NS - 2) into slot j mod (NS - 2) of this
    // wave (K ids, then V ids); those of steps 1 .. NS - 3 are fetched here.
    char *const idk_slots = lds + 2 * NS * C::kTileBytes + (2 * wave) * (C::kIdSlots * kIdSlotBytes);
    char *const idv_slots = idk_slots + C::kIdSlots * kIdSlotBytes;
    if (copier) {
#pragma unroll
        for (int t = 0; t < NS - 1; t++) {
            cpk.copy(prefill_page_id<D>(pages, n_pages, t_begin + t, pg), t);
            cpv.copy(prefill_page_id<D>(pages, n_pages, t_begin + t, pg), t);
        }
        cpk.copy(prefill_page_id<D>(pages, n_pages, t_begin + NS - 1, pg), NS - 1);
        idk_cur = prefill_page_id<D>(pages, n_pages, t_begin + NS, pg);
        idv_cur = prefill_page_id<D>(pages, n_pages, t_begin + NS - 1, pg);
#pragma unroll
        for (int t = 1; t < C::kIdSlots; t++) {
            page_id_fetch(pages + min((t_begin + t + NS) * C::kTilePages + pg, n_pages - 1), idk_slots + t * kIdSlotBytes);
            page_id_fetch(pages + min((t_begin + t + NS - 1) * C::kTilePages + pg, n_pages - 1), idv_slots + t * kIdSlotBytes);
        }
        wait_all_loads();
#pragma unroll
        for (int t = 0; t < NS - 1; t++)
            if ((t_begin + t + 1) * C::kTileTokens > kv_len) prefill_fix_tail<D>(lds_v + t * C::kTileBytes, t_begin + t, pg, lane, kv_len);
    }
    __syncthreads();
    x8 kf[KS];     // K fragments of the half whose scores are computed next
    x8 vf[2][MT];  // V^T fragments of the half whose P V product comes next
    x8 pb[2];      // probabilities of that half (B operands, one per page)
    f32x16 sc, sn;
    W::load_k((lds_cptr)(lds_k + k_lane_off), 0, kf);
    W::qk(kf, qreg, sc);
    W::load_k((lds_cptr)(lds_k + k_lane_off), 1, kf);
    // the first phase has no earlier half to accumulate: give its P V product zero probabilities
    W::load_v((lds_cptr)(lds_v + v_lane_off), 0, vf);
#pragma unroll
    for (int b = 0; b < 2; b++)
#pragma unroll
        for (int e = 0; e < 8; e++) pb[b][e] = (el)0.f;
    if (t_begin * C::kTileTokens + 31 > wave_pmin) W::causal_mask(sc, t_begin * C::kTileTokens, hh, p_abs);
    m_run = next_reference_max(m_run, W::row_max(sc) * c_log2);  // the first half-tile's true maxima
    float psum = 0.f;  // this lane's sum of the probabilities just computed

    // After the probabilities `pb` of a half-tile with scores `s_pb`, and after the product of the half
    // before it: the reference maximum served if no lane's sum got out of hand; else (rare, wave-uniform
    // branch) move it for the rows that need it, bring O and l to the new reference and compute the
    // probabilities again.
    auto settle = [&](const f32x16 &s_pb) {
        if (__builtin_amdgcn_ballot_w64(!(psum <= kSumLimit)) != 0) {
            const float m_new = next_reference_max(m_run, W::row_max(s_pb) * c_log2);
            const float a = fast_exp2(m_run - m_new);
            m_run = m_new;
            l_run *= a;
#pragma unroll
            for (int c = 0; c < MT; c++)
#pragma unroll
                for (int r = 0; r < 16; r++) o[c][r] *= a;
            W::probs(s_pb, c_log2, m_run, pb, psum);
        }
        l_run += psum;
    };

    // One phase, for half-tile h: `cur` holds its scores S(h), `kf` the K fragments of half h + 1, `vf` /
    // `pb` the V^T fragments and probabilities of half h - 1.
    //   matrix cores:  S(h+1) = K(h+1) Q^T  (QK),   O += V(h-1)^T P(h-1)^T
    //   vector ALU:    P(h) = 2^(S(h) c - m)  under those MFMAs; then `settle`
    //   LDS:           every MFMA is followed by the read that refills its operand register for the next
    //                  phase: K fragments of half h + 2 (KREAD), V^T fragments of half h
    // MASK: half h + 1 may reach past a row's own position or past the last token.  Without MASK the
    // phase is, apart from the branch in `settle`, one straight line of code.
    auto phase = [&](lds_cptr v_h, int hv, lds_cptr k_after, int hk, f32x16 &cur, f32x16 &nxt, int tok_nxt, auto mask_tag,
                     auto qk_tag, auto kread_tag) {
        constexpr bool MASK = decltype(mask_tag)::value, QK = decltype(qk_tag)::value, KREAD = decltype(kread_tag)::value;
        if (QK) W::qk(kf, qreg, nxt);
        if (KREAD) W::load_k(k_after, hk, kf);
        W::pv(vf, pb, o);
        W::load_v(v_h, hv, vf);
        W::probs(cur, c_log2, m_run, pb, psum);
        if (MASK && QK) W::causal_mask(nxt, tok_nxt, hh, p_abs);
        // the probabilities are used by the next phase: have them computed in this one
        asm volatile("" : "+v"(pb[0]), "+v"(pb[1]), "+v"(psum));
        if (!MASK && QK && KREAD) {
            // per MFMA: the read that refills its operand; under ten of the phase's MFMAs, from the sixth on, softmax
            // work for two elements each (measured against it on a long sweep: under the first ten 1.2 % slower,
            // under the last ten 0.6 %, one element under every MFMA 2 %, three under the first eight 3.5 %)
            constexpr int kMfma = KS + 2 * MT;
            constexpr int kProb = kMfma >= 16 ? 10 : kMfma - 2, kFirst = kMfma - kProb - 1, kPer = (16 + kProb - 1) / kProb;
#pragma unroll
            for (int g = 0; g < kMfma; g++) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                if (g >= kFirst && g < kFirst + kProb) {
                    __builtin_amdgcn_sched_group_barrier(0x002, kPer, 0);
                    __builtin_amdgcn_sched_group_barrier(0x400, kPer, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, kPer, 0);
                }
            }
        }
        settle(cur);
    };
    // One step for tile t_begin + j, which lives in stage s0 = j mod NS: `sc` holds the scores of its first
    // half, `kf` the K fragments of its second half.  NEXT: tile j + 1 exists.
    int s0 = 0, id_slot = 0;  // stage of the step's tile; slot that receives the page id fetched in the step (j mod (NS - 2))
    auto step = [&](int j, auto mask_tag, auto next_tag) {
        constexpr bool NEXT = decltype(next_tag)::value;
        const int tile = t_begin + j;
        const int s1 = s0 == NS - 1 ? 0 : s0 + 1, sm1 = s0 == 0 ? NS - 1 : s0 - 1;
        lds_cptr k_nxt = (lds_cptr)(lds_k + s1 * C::kTileBytes + k_lane_off);
        lds_cptr v_cur = (lds_cptr)(lds_v + s0 * C::kTileBytes + v_lane_off);
        // have both operand addresses in registers here, outside the scheduled regions below
        asm volatile("" : "+v"(k_nxt), "+v"(v_cur));
        __syncthreads();  // every wave is done with step j - 1; the copies issued in step j - (NS - 1) are visible
        if (NEXT && copier) {
            // first the page ids for the copies of step j + NS - 2, then this step's copies: K(j+NS) replaces K(j),
            // V(j+NS-1) replaces V(j-1).  Past the end of the range the page index is clamped and the copy
            // is never read.
            page_id_fetch(pages + min((tile + NS - 2 + NS) * C::kTilePages + pg, n_pages - 1), idk_slots + id_slot * kIdSlotBytes);
            page_id_fetch(pages + min((tile + NS - 2 + NS - 1) * C::kTilePages + pg, n_pages - 1), idv_slots + id_slot * kIdSlotBytes);
            cpk.copy(idk_cur, s0);
            cpv.copy(idv_cur, sm1);
        }
        const std::true_type yes;
        phase(v_cur, 0, k_nxt, 0, sc, sn, tile * C::kTileTokens + 32, mask_tag, yes, next_tag);
        phase(v_cur, 1, k_nxt, 1, sn, sc, (tile + 1) * C::kTileTokens, mask_tag, next_tag, next_tag);
        if (NEXT && copier) {
            // loads return in order: all but the copies of the last NS - 2 steps and the page ids fetched
            // after those for step j + 1 have landed, i.e. those page ids and the copies of step j - (NS - 2)
            wait_loads_but<(NS - 2) * (2 * C::kRuns + 2) - 2>();
            id_slot = id_slot == C::kIdSlots - 1 ? 0 : id_slot + 1;  // slot of step j + 1
            idk_cur = page_id_read(idk_slots + id_slot * kIdSlotBytes, lane);
            idv_cur = page_id_read(idv_slots + id_slot * kIdSlotBytes, lane);
            if (decltype(mask_tag)::value && (tile + 2) * C::kTileTokens > kv_len)
                prefill_fix_tail<D>(lds_v + s1 * C::kTileBytes, tile + 1, pg, lane, kv_len);
        }
        s0 = s1;
    };
    {
        const std::true_type yes;
        const std::false_type no;
        // steps 0 .. n_plain - 1 prepare tiles that lie wholly at or before every row's position
        // and before the last token: tile t needs no mask if (t + 1) * 64 - 1 <= wave_pmin
        const int n_plain = max(0, min(n_sweep - 1, (wave_pmin + 1) / C::kTileTokens - t_begin - 1));
        int j = 0;
        for (; j < n_plain; j++) step(j, no, yes);
        for (; j + 1 < n_sweep; j++) step(j, yes, yes);
        step(j, yes, no);
    }
    // the product of the last half
    W::pv(vf, pb, o);

    float l = half_swap_sum(l_run);
    if (p_slot >= 0) {
        // A piece of a cut item: every lane leaves its unnormalised accumulators, and the rows' running maximum
        // (log2 domain) and sum, in the piece's region of the workspace as they lie in registers; rows that see no
        // key of this piece carry (m, l, o) = (-1e30, 0, 0) and get weight 0 in the combination.
        float *const region = A.ws_pieces + (int64_t)(p_slot + pc[PP_C]) * PiecePartial<D>::kFloats;
        PiecePartial<D>::store(region, wave, lane, o, m_run, l, A.fused != 0);
        if (!A.fused) return;
        // The last of the item's pieces to get here combines them all (the others leave; nobody waits).  Every
        // wave waits for its own stores to complete, the workgroup meets, one thread counts the arrival.
        stores_done();
        __syncthreads();  // every wave has left the sweep: LDS is free
        int *const arrived = reinterpret_cast<int *>(lds);
        int32_t *const counter = A.counters + pc[PP_COUNTER];
        if (tid == 0) *arrived = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (*arrived != p_k - 1) return;
        if (tid == 0) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // for the next launch
        PiecePartial<D>::template combine<true>(A.ws_pieces + (int64_t)p_slot * PiecePartial<D>::kFloats, p_k, wave, lane, o, l);
    }
    if (row_valid) prefill_write_rows<D, E>(A.out + row_off, o, l, hh);
}

// ------------------------------------------------------------------------------------
// Decode branch: one wavefront = one (sequence, KV head, KV split); all G query heads of
// the group ride in the N dimension of the MFMA so K/V are read once per KV head.
// ------------------------------------------------------------------------------------
// Lane l: head column j = l % 16, token group g = l / 16.  Per page:
//   S^T[token][head] = sum_d K[token][d] Q[head][d]   16x16x32, D/32 steps; lane gets tokens 4g..4g+3
//   O^T[d][head]    += sum_token V^T[d][token] P^T[token][head]   16x16x16, contraction over the page's
//                      16 tokens: lane feeds tokens 4g..4g+3
// Pages resident in registers per wave (NS): one being consumed, the rest in flight.  Two keep the
// decode-only kernel within 168 VGPRs (three waves per SIMD; a third stage spills there).  In a launch
// with a prefill chunk the decode workgroups are one per compute unit and share the chip with the chunk, so
// a few units must carry the whole decode stream: there a wave keeps kMixedDecodeStages - 1 pages in flight.
constexpr int kDecodeStages = 2;
constexpr int kMixedDecodeStages = 4;

template <int D>
struct DecodePage {  // K and V of one page, in MFMA A-operand registers
    u32x4 k[D / 32];
    u32x2 v[D / 16];
};

// KV pages are read exactly once per launch, by one wavefront: stream them past the caches.
// When the attention kernel also does the append (a batch of decodes: tc_mixed_attention_append), the newest
// token of a sequence (index tn of the last page of its last KV split) may not be in the pool yet when that
// page is fetched: the rows are stored by the last workgroups of the same launch (append_decode_rows),
// and nobody waits for them.  The wavefront that runs the split therefore takes the token's K and V from this
// iteration's rows and puts them in the place of what the fetch found in that slot.  (Storing the token from
// here, scattered through a launch that streams K/V at the HBM limit, cost 40-60 us on 512 sequences where the
// append kernel needs 14, and so did storing them from workgroups at the front of the launch; from workgroups at its
// back, which run while the grid drains and after nearly every page has been read, they cost less than the launch they replace.)
template <int D>
__device__ __forceinline__ void decode_take_new_token(const AttnArgs &A, int kvh, int qrow, int tn, int j, int g, DecodePage<D> &st) {
    const uint16_t *kn = A.k_new + ((int64_t)qrow * A.Hkv + kvh) * D;
    const uint16_t *vn = A.v_new + ((int64_t)qrow * A.Hkv + kvh) * D;
    if (j == tn) {  // K: this lane holds the 8-element pieces 4 kk + g of token j
#pragma unroll
        for (int kk = 0; kk < D / 32; kk++) st.k[kk] = *reinterpret_cast<const u32x4 *>(kn + (4 * kk + g) * 8);
    }
    if (g == (tn >> 2)) {  // V: this lane holds tokens 4 g .. 4 g + 3 of the elements 16 c + j
        const int e = tn & 3;
#pragma unroll
        for (int c = 0; c < D / 16; c++) {
            const uint32_t val = vn[16 * c + j];
            u32x2 w = st.v[c];
            const uint32_t keep = (e & 1) ? 0x0000FFFFu : 0xFFFF0000u, put = (e & 1) ? val << 16 : val;
            if (e >> 1) w[1] = (w[1] & keep) | put; else w[0] = (w[0] & keep) | put;
            st.v[c] = w;
        }
    }
}

// The append of a batch of decodes, done by the last workgroups of the attention launch: thread = (sequence, KV head,
// 8-element piece) copies the piece of the new token's K and scatters the piece of its V (token-minor pool), four per
// thread.  `segments`: the plan's append segments, one per sequence here (one token each).
template <int D>
__device__ __forceinline__ void append_decode_rows(const AttnArgs &A, const int32_t *__restrict__ segments, int n_rows, int wg) {
    constexpr int CH = D / 8, kPerThread = 4;
    const int total = n_rows * A.Hkv * CH;
#pragma unroll
    for (int i = 0; i < kPerThread; i++) {
        const int x = (wg * kPerThread + i) * (int)blockDim.x + (int)threadIdx.x;
        if (x < total) {
            const int c = x % CH, h = (x / CH) % A.Hkv;
            const int32_t *seg = segments + (int64_t)(x / (CH * A.Hkv)) * kAppendInts;
            const int row = seg[0], tok = seg[2];
            const int64_t tile = ((int64_t)seg[3] * A.Hkv + h) * (int64_t)(kBlock * D);
            const int64_t src = ((int64_t)row * A.Hkv + h) * D + c * 8;
            *reinterpret_cast<u32x4 *>(A.k_pool + tile + ((int64_t)c * kBlock + tok) * 8) = *reinterpret_cast<const u32x4 *>(A.k_new + src);
            const u32x4 v = *reinterpret_cast<const u32x4 *>(A.v_new + src);
            uint16_t *dst = A.v_pool + tile + (int64_t)(c * 8) * kBlock + v_slot(tok);
#pragma unroll
            for (int e = 0; e < 8; e++) dst[e * kBlock] = (uint16_t)(v[e >> 1] >> ((e & 1) * 16));
        }
    }
}

template <int D>
__device__ __forceinline__ void decode_fetch(const AttnArgs &A, int kvh, int id, int j, int g, DecodePage<D> &st) {
    const int64_t tile_elems = (int64_t)kBlock * D;
    const uint16_t *kb = A.k_pool + ((int64_t)id * A.Hkv + kvh) * tile_elems;
    const uint16_t *vb = A.v_pool + ((int64_t)id * A.Hkv + kvh) * tile_elems;
#pragma unroll
    for (int kk = 0; kk < D / 32; kk++)
        st.k[kk] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(kb + ((4 * kk + g) * kBlock + j) * 8));
#pragma unroll
    for (int c = 0; c < D / 16; c++)
        st.v[c] = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(vb + (16 * c + j) * kBlock + v_slot(4 * g)));
}

// One page: S^T = K Q^T (16 tokens x 16 head columns, contraction over D), online softmax over the
// 16 tokens, O^T += V^T P^T (contraction over the page's 16 tokens).
template <int D, class E>
__device__ __forceinline__ void decode_consume(const AttnArgs &A, DecodePage<D> &st, const typename E::x8 (&qreg)[D / 32],
                                               int n_valid, int g, f32x4 (&o)[D / 16], float &m_run, float &l_run) {
    using x8 = typename E::x8;
    using x4 = typename E::x4;
    using el = typename E::t;
    constexpr int KS = D / 32, MT = D / 16;
    // two accumulators: the second half of the head dimension does not wait for the first
    f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f}, s_hi = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < KS / 2; kk++) {
        s = E::mfma16(__builtin_bit_cast(x8, st.k[kk]), qreg[kk], s);
        s_hi = E::mfma16(__builtin_bit_cast(x8, st.k[kk + KS / 2]), qreg[kk + KS / 2], s_hi);
    }
    s += s_hi;
    if (n_valid < kBlock) {  // the split ends inside this page: mask scores, make V finite
#pragma unroll
        for (int r = 0; r < 4; r++) s[r] = (4 * g + r < n_valid) ? s[r] : -INFINITY;
#pragma unroll
        for (int c = 0; c < MT; c++) {
            u32x2 w = st.v[c];
            if (4 * g + 0 >= n_valid) w[0] &= 0xFFFF0000u;
            if (4 * g + 1 >= n_valid) w[0] &= 0x0000FFFFu;
            if (4 * g + 2 >= n_valid) w[1] &= 0xFFFF0000u;
            if (4 * g + 3 >= n_valid) w[1] &= 0x0000FFFFu;
            st.v[c] = w;
        }
    }
    // As in the prefill branch the reference maximum of a head column (log2 domain) is kept while it serves: the page's
    // probabilities are computed against it as it is, and only when a lane's sum of its four gets out of hand (one
    // of them is above 2^11; the test also catches the first page, whose reference is -1e30, and NaN) does the wave, in
    // a uniform branch, find the page's true maxima, move the reference of the columns that need it, bring O and l
    // to it and compute the probabilities again.  The common page has no reduction across lanes and no rescaling:
    // beside a prefill chunk the decode branch runs on few compute units and is bound by its own instructions.
    x4 pb;
    float psum = 0.f;
#pragma unroll
    for (int r = 0; r < 4; r++) {
        const float pv = fast_exp2(__builtin_fmaf(s[r], A.scale_log2, -m_run));
        psum += pv;
        pb[r] = (el)pv;
    }
    if (__builtin_amdgcn_ballot_w64(!(psum <= kSumLimit)) != 0) {
        float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
        mx = fmaxf(mx, xor_lanes(mx, 16));
        mx = half_swap_max(mx);
        const float m_new = next_reference_max(m_run, mx * A.scale_log2);
        const float alpha = fast_exp2(m_run - m_new);
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int c = 0; c < MT; c++) o[c] *= alpha;
        psum = 0.f;
#pragma unroll
        for (int r = 0; r < 4; r++) {
            const float pv = fast_exp2(__builtin_fmaf(s[r], A.scale_log2, -m_new));
            psum += pv;
            pb[r] = (el)pv;
        }
    }
    l_run += psum;
#pragma unroll
    for (int c = 0; c < MT; c++) o[c] = E::mfma16k16(__builtin_bit_cast(x4, st.v[c]), pb, o[c]);
}

// The splits of one (sequence, KV head) that share a workgroup form a team (consecutive waves): the
// members leave their (m, l, O) in LDS and the team's first wave combines them, in wave order, with its
// own and writes the output rows, or one partial result if the (sequence, KV head) has more teams.
// Bytes of LDS a decode workgroup of `waves` waves needs for that.
__host__ __device__ constexpr size_t decode_team_lds_bytes(int waves, int G, int D) { return (size_t)waves * G * (D + 2) * sizeof(float); }

template <int D, class E, int NS>
__device__ void decode_item(const AttnArgs &A, const int32_t *__restrict__ it, float *team_lds, int wg_waves) {
    using x8 = typename E::x8;
    using x4 = typename E::x4;
    using el = typename E::t;
    constexpr int KS = D / 32;  // k-steps of K Q^T
    constexpr int MT = D / 16;  // 16-row tiles of O^T
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));  // may be called in a loop: derive the per-lane values afresh for every item (see prefill_item)
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15, g = lane >> 4;
    const int kvh = it[DC_KVH], t0 = it[DC_BEGIN], t1 = it[DC_END], qrow = it[DC_QROW], slot = it[DC_SLOT];
    const int team_n = it[DC_TEAM] & 15, team_pos = (it[DC_TEAM] >> 4) & 7, merge_item = (it[DC_TEAM] >> 8) - 1;
    // the split ends with the sequence's newest token and this launch is the one that stores it
    const bool takes_new = (it[DC_TEAM] & kTeamTailBit) && A.k_new != nullptr;
    const int G = A.G;
    const int n_tok = t1 - t0;  // 0: a padding item, which only takes part in the barrier

    f32x4 o[MT];
#pragma unroll
    for (int c = 0; c < MT; c++) o[c] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -1e30f, l_run = 0.f;

    if (n_tok > 0) {
        const int page0 = t0 / kBlock;
        const int n_pg = (n_tok + kBlock - 1) / kBlock;  // 1..64
        const int32_t *pages = A.pages + it[DC_PAGEOFF] + page0;
        const int my_page = pages[min(lane, n_pg - 1)];  // lane i holds the id of page i of the split

        x8 qreg[KS];
        const int64_t q_off = ((int64_t)qrow * A.Hq + kvh * G + min(j, G - 1)) * D;
#pragma unroll
        for (int kk = 0; kk < KS; kk++) {
            u32x4 w = *reinterpret_cast<const u32x4 *>(A.q + q_off + (4 * kk + g) * 8);
            if (j >= G) w = u32x4{0u, 0u, 0u, 0u};
            qreg[kk] = __builtin_bit_cast(x8, w);
        }

        // A ring of NS register stages, one page each: while page i is consumed the loads of pages
        // i+1 .. i+NS-1 are in flight.
        DecodePage<D> st[NS];
#pragma unroll
        for (int u = 0; u < NS - 1; u++)
            if (u < n_pg) decode_fetch<D>(A, kvh, __builtin_amdgcn_readlane(my_page, u), j, g, st[u]);
        // Main part: every page consumed here is full and every fetch is of a page of the split, so the body
        // has no branch around the loads and the compiler's wait before a stage's first use counts exactly
        // the loads issued after it.  (With a conditional fetch the wait has to be right for the path
        // without it, and then also waits for the page just requested: one page in flight instead of NS - 1.)
        int pp = 0;
        for (; pp + 2 * (NS - 1) < n_pg; pp += NS) {
#pragma unroll
            for (int u = 0; u < NS; u++) {
                decode_fetch<D>(A, kvh, __builtin_amdgcn_readlane(my_page, pp + u + NS - 1), j, g, st[(u + NS - 1) % NS]);
                decode_consume<D, E>(A, st[u], qreg, kBlock, g, o, m_run, l_run);
            }
        }
        // The last pages (at most 2 NS - 2): fetch while there is a page left, the last one may be partial.
        for (; pp < n_pg; pp += NS) {
#pragma unroll
            for (int u = 0; u < NS; u++) {
                const int cur = pp + u;
                if (cur < n_pg) {
                    const int nxt = cur + NS - 1;
                    if (nxt < n_pg) decode_fetch<D>(A, kvh, __builtin_amdgcn_readlane(my_page, nxt), j, g, st[(u + NS - 1) % NS]);
                    if (takes_new && cur == n_pg - 1)
                        decode_take_new_token<D>(A, kvh, qrow, (n_tok - 1) & (kBlock - 1), j, g, st[u]);
                    decode_consume<D, E>(A, st[u], qreg, n_tok - cur * kBlock, g, o, m_run, l_run);
                }
            }
        }
        l_run += xor_lanes(l_run, 16);
        l_run = half_swap_sum(l_run);
    }

    // ---- team: members (positions 1 ..) hand their result to the first wave through LDS
    // LDS: O^T of every wave [waves][G][D], then (m, l) [waves][G][2]; a lane reads back the elements it owns
    float *const my_o = team_lds + (size_t)wave * G * D;
    float *const my_ml = team_lds + (size_t)wg_waves * G * D + (size_t)wave * G * 2;
    if (team_pos > 0 && j < G) {
        float *dst = my_o + j * D + 4 * g;
#pragma unroll
        for (int c = 0; c < MT; c++) *reinterpret_cast<f32x4 *>(dst + 16 * c) = o[c];
        if (g == 0) {
            my_ml[2 * j] = m_run;
            my_ml[2 * j + 1] = l_run;
        }
    }
    __syncthreads();  // executed once by every wave of a decode workgroup, for every unit of items it runs
    if (team_pos > 0 || n_tok == 0) return;
    const int jc = min(j, G - 1);  // head columns past G are padding: they follow column G - 1 and store nothing
    for (int i = 1; i < team_n; i++) {
        const float m_i = my_ml[(i * G + jc) * 2], l_i = my_ml[(i * G + jc) * 2 + 1];
        const float m_new = fmaxf(m_run, m_i);
        const float a = fast_exp2(m_run - m_new), b = fast_exp2(m_i - m_new);
        m_run = m_new;
        l_run = l_run * a + l_i * b;
        const float *src = my_o + (size_t)i * G * D + jc * D + 4 * g;
#pragma unroll
        for (int c = 0; c < MT; c++) o[c] = o[c] * a + *reinterpret_cast<const f32x4 *>(src + 16 * c) * b;
    }
    if (slot < 0) {
        if (j < G) {
            const float inv = 1.f / l_run;
            uint16_t *dst = A.out + ((int64_t)qrow * A.Hq + kvh * G + j) * D + 4 * g;
#pragma unroll
            for (int c = 0; c < MT; c++) {
                x4 w;
#pragma unroll
                for (int e = 0; e < 4; e++) w[e] = (el)(o[c][e] * inv);
                *reinterpret_cast<x4 *>(dst + 16 * c) = w;
            }
        }
        return;
    }
    if (j < G) {
        float *dst = A.ws_o + ((int64_t)slot * G + j) * D + 4 * g;
        float *ml = A.ws_ml + ((int64_t)slot * G + j) * 2;
        if (A.fused) {
#pragma unroll
            for (int c = 0; c < MT; c++) {
                peer_store2(dst + 16 * c, o[c][0], o[c][1]);
                peer_store2(dst + 16 * c + 2, o[c][2], o[c][3]);
            }
            if (g == 0) peer_store2(ml, m_run, l_run);
        } else {
            // partial results are written once and read once: stream them past the caches (plain
            // stores of these 2 KiB per split measured 3 % less bandwidth on a batch of decodes)
#pragma unroll
            for (int c = 0; c < MT; c++) __builtin_nontemporal_store(o[c], reinterpret_cast<f32x4 *>(dst + 16 * c));
            if (g == 0) {
                ml[0] = m_run;
                ml[1] = l_run;
            }
        }
    }
    if (!A.fused) return;
    // the last team of the (sequence, KV head) to get here combines the partial results of all of them
    const int32_t *mg = A.merge + (int64_t)merge_item * kItemInts;
    int32_t *const counter = A.counters + mg[MG_COUNTER];
    if (!arrive_is_last(counter, mg[MG_NSPLIT], lane == 0)) return;
    for (int h = 0; h < G; h++)
        merge_row<D, E, true>(A.ws_o, A.ws_ml, mg[MG_SLOT0], mg[MG_NSPLIT], G, h, A.out + ((int64_t)qrow * A.Hq + kvh * G + h) * D, lane);
    if (lane == 0) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

#ifdef TC_WG_TRACE
// Tracing build (python -m paper_2508_01989_amd.build --trace): every workgroup of the attention kernel leaves the time
// it started, the time its prefill pieces were done and the time it ended (100 MHz counter), and where it ran.
constexpr int kTraceWorkgroups = 16384;
__device__ long long g_wg_trace[kTraceWorkgroups * 4];
#endif

struct AttnScalars {
    int n_prefill, n_decode;
    int Hq, Hkv, G;
    int fused;
    int queue;
    int n_partials;
    int n_front, n_append_rows;  // a batch of decodes whose rows this launch stores: the workgroups (the last of the grid) that do it, rows
    float scale_log2;
};

// The work lists and the page table are separate const __restrict__ kernel arguments (not struct
// members) so that the compiler knows they are never written and can fetch them with
// scalar loads.  WAVES = 8: batches with a prefill chunk (one workgroup per compute unit, up to 256
// registers per wave); WAVES = 4: decode-only batches (three workgroups per compute unit).
// Workgroups [0, n_prefill) run the prefill pieces the plan gave them, one after the other; the rest run
// decode items, one per wave.
template <int D, class E, int WAVES>
__global__ void __launch_bounds__(WAVES * 64, WAVES == kMixedWaves ? 1 : kDecodeWgPerCu)
    mixed_attention_kernel(uint16_t *k_pool, uint16_t *v_pool, const uint16_t *__restrict__ q, const uint16_t *__restrict__ k_new,
                           const uint16_t *__restrict__ v_new, uint16_t *__restrict__ out, const int32_t *__restrict__ pages,
                           const int32_t *__restrict__ prefill, const int32_t *__restrict__ pieces,
                           const int32_t *__restrict__ wg_first, const int32_t *__restrict__ decode,
                           const int32_t *__restrict__ merge, const int32_t *__restrict__ append, int32_t *counters, float *ws,
                           const AttnScalars sc) {
    extern __shared__ __align__(16) char lds[];
#ifdef TC_WG_TRACE
    const long long t_start = __builtin_amdgcn_s_memrealtime();
    long long t_mid = t_start;
#endif
    AttnArgs A;
    A.k_pool = k_pool; A.v_pool = v_pool; A.q = q; A.k_new = k_new; A.v_new = v_new; A.out = out; A.pages = pages; A.prefill = prefill;
    A.pieces = pieces; A.wg_first = wg_first; A.decode = decode; A.merge = merge; A.counters = counters;
    // workspace: decode partials [n_partials][G][D], their (max, sum) pairs [n_partials][G][2], then the piece regions
    A.ws_o = ws; A.ws_ml = ws + (int64_t)sc.n_partials * sc.G * D; A.ws_pieces = A.ws_ml + (int64_t)sc.n_partials * sc.G * 2;
    A.n_prefill = sc.n_prefill; A.n_decode = sc.n_decode; A.Hq = sc.Hq; A.Hkv = sc.Hkv; A.G = sc.G; A.fused = sc.fused; A.queue = sc.queue;
    A.scale_log2 = sc.scale_log2;
    constexpr int NS = WAVES == kMixedWaves ? kMixedDecodeStages : kDecodeStages;
    if constexpr (WAVES == kDecodeWaves) {
        const int first_append_wg = (int)gridDim.x - sc.n_front;
        if ((int)blockIdx.x >= first_append_wg) {
            append_decode_rows<D>(A, append, sc.n_append_rows, (int)blockIdx.x - first_append_wg);
            return;
        }
    }
    const int wg = (int)blockIdx.x;
    if (WAVES == kMixedWaves && (int)blockIdx.x < A.n_prefill) {
        if constexpr (WAVES == kMixedWaves) {
            const int32_t *pc = pieces + (int64_t)wg_first[blockIdx.x] * kItemInts;
            for (;;) {
                prefill_item<D, E>(A, prefill + (int64_t)pc[PP_ITEM] * kItemInts, pc, lds);
                if (pc[PP_LAST]) break;
                pc += kItemInts;
                __syncthreads();  // the next piece's tile copies reuse the LDS
            }
        }
    } else if (WAVES != kMixedWaves || A.queue < 0) {
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const int idx = (wg - A.n_prefill) * WAVES + wave;
        // the decode items fill whole workgroups (padding items at the end of some): every wave gets one
        if (idx < A.n_decode) decode_item<D, E, NS>(A, decode + (int64_t)idx * kItemInts, reinterpret_cast<float *>(lds), WAVES);
    }
#ifdef TC_WG_TRACE
    t_mid = __builtin_amdgcn_s_memrealtime();
#endif
    if constexpr (WAVES == kMixedWaves) {
        if (A.queue >= 0) {
        // Decode queue (the launch has no more workgroups than the chip has compute units, all resident from the
        // start).  The decode items are handed out in units of one workgroup's worth (WAVES items, teams included)
        // through a counter: the workgroups launched for the decode branch draw from the start, the prefill
        // workgroups join when their pieces are done, and everybody leaves when the counter has passed the last unit,
        // so that whichever compute unit is free carries the decode stream and no workgroup waits for another.
        // (Left to the hardware, decode workgroups beyond the first round were not started on the units the first
        // round had freed until the prefill workgroups ended.  Handing out single items to single waves, with the
        // splits of a pair combined by the last to arrive, measured slower than units with their teams.)
        // The workgroup that leaves last puts both counters back to zero for the next launch.
        int *const drawn = reinterpret_cast<int *>(lds + PrefillCfg<D>::kQueueSlot);
        int32_t *const next_unit = A.counters + A.queue, *const gone = next_unit + 1;
        const int n_units = A.n_decode / WAVES;
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        for (;;) {
            __syncthreads();  // the unit before (or the last prefill piece) is done with the LDS
            if (threadIdx.x == 0) *drawn = __hip_atomic_fetch_add(next_unit, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            const int unit = *drawn;
            if (unit >= n_units) break;
            decode_item<D, E, NS>(A, decode + ((int64_t)unit * WAVES + wave) * kItemInts, reinterpret_cast<float *>(lds), WAVES);
        }
        if (threadIdx.x == 0 && __hip_atomic_fetch_add(gone, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (int)gridDim.x - 1) {
            __hip_atomic_store(next_unit, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(gone, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        }
    }
#ifdef TC_WG_TRACE
    __syncthreads();
    if (threadIdx.x == 0 && blockIdx.x < kTraceWorkgroups) {
        unsigned hw, xcc;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
        long long *t = g_wg_trace + (long long)blockIdx.x * 4;
        t[0] = t_start;
        t[1] = __builtin_amdgcn_s_memrealtime();
        t[2] = ((long long)xcc << 32) | hw;
        t[3] = (((int)blockIdx.x < sc.n_prefill) ? 0 : 1) | ((t_mid - t_start) << 8);
    }
#endif
}

// ------------------------------------------------------------------------------------
// Split-KV merge as a launch of its own (the two-call form; the fused kernel does the same inside)
// ------------------------------------------------------------------------------------
// One workgroup per split decode (sequence, KV head) pair; one wavefront per query head.
template <int D, class E>
__global__ void __launch_bounds__(256) split_merge_kernel(const int32_t *__restrict__ items, const float *__restrict__ ws_o,
                                                          const float *__restrict__ ws_ml, uint16_t *__restrict__ out,
                                                          int Hq, int G) {
    const int32_t *it = items + (int64_t)blockIdx.x * kItemInts;
    const int kvh = it[MG_KVH], qrow = it[MG_QROW], ns = it[MG_NSPLIT], slot0 = it[MG_SLOT0];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int j = wave; j < G; j += 4) merge_row<D, E, false>(ws_o, ws_ml, slot0, ns, G, j, out + ((int64_t)qrow * Hq + kvh * G + j) * D, lane);
}

// One workgroup per cut prefill item, with the lane-to-row map of the prefill branch: the lanes read the pieces'
// partial results back as the pieces' lanes left them and write the item's output rows.
template <int D, class E>
__global__ void __launch_bounds__(kMixedWaves * 64) prefill_merge_kernel(const int32_t *__restrict__ items, const int32_t *__restrict__ prefill,
                                                                          const float *__restrict__ ws_pieces, uint16_t *__restrict__ out,
                                                                          int Hq, int G) {
    const int32_t *mg = items + (int64_t)blockIdx.x * kItemInts;
    const int32_t *it = prefill + (int64_t)mg[MG_ITEM] * kItemInts;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n = lane & 31, hh = lane >> 5;
    const int kvh = it[PF_KVH], pos0 = it[PF_POS0], npos = it[PF_NPOS], qrow0 = it[PF_QROW0];
    const int R = wave * 32 + n;
    f32x16 o[D / 32];
    float l;
    PiecePartial<D>::template combine<false>(ws_pieces + (int64_t)mg[MG_SLOT0] * PiecePartial<D>::kFloats, mg[MG_NSPLIT], wave, lane, o, l);
    if (R < npos * G) prefill_write_rows<D, E>(out + ((int64_t)(qrow0 + pos0 + R / G) * Hq + kvh * G + R % G) * D, o, l, hh);
}

// ------------------------------------------------------------------------------------
// Plan buffers
// ------------------------------------------------------------------------------------
const char *hip_error_text(int err) { return hipGetErrorString((hipError_t)err); }

int begin_plan_host(tc_plan *p, size_t n) {
    if (p->upload_event) {
        hipError_t e = hipEventSynchronize((hipEvent_t)p->upload_event);
        if (e != hipSuccess) return (int)e;
    }
    if (n <= p->host_cap) return 0;
    const size_t cap = std::max<size_t>(n + n / 2, 4096);
    int32_t *fresh = nullptr;
    if (p->on_device) {
        hipError_t e = hipHostMalloc((void **)&fresh, cap * sizeof(int32_t), hipHostMallocDefault);
        if (e != hipSuccess) return (int)e;
    } else {
        fresh = (int32_t *)std::malloc(cap * sizeof(int32_t));
        if (!fresh) return (int)hipErrorOutOfMemory;
    }
    if (p->host) {
        if (p->host_pinned) (void)hipHostFree(p->host); else std::free(p->host);
    }
    p->host = fresh;
    p->host_cap = cap;
    p->host_pinned = p->on_device;
    return 0;
}

// Copy the host image to the device on `stream`.  The device buffer grows when a work list is larger than
// any before it and is otherwise reused: a serving loop that keeps one plan object allocates nothing per
// iteration.  (Growing frees the old buffer, which waits for the device to finish whatever still reads it.)
int upload_plan(tc_plan *p, void *stream) {
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return (int)e;
    if (p->device >= 0 && p->device != device) return (int)hipErrorInvalidDevice;
    p->device = device;
    if (p->host_n > p->dev_cap) {
        if (p->dev) (void)hipFree(p->dev);
        p->dev = nullptr;
        p->dev_cap = 0;
        e = hipMalloc((void **)&p->dev, p->host_cap * sizeof(int32_t));
        if (e != hipSuccess) { p->dev = nullptr; return (int)e; }
        p->dev_cap = p->host_cap;
    }
    if (!p->upload_event) {
        hipEvent_t ev;
        e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
        if (e != hipSuccess) return (int)e;
        p->upload_event = ev;
    }
    e = hipMemcpyAsync(p->dev, p->host, p->host_n * sizeof(int32_t), hipMemcpyHostToDevice, (hipStream_t)stream);
    if (e != hipSuccess) return (int)e;
    return (int)hipEventRecord((hipEvent_t)p->upload_event, (hipStream_t)stream);
}

void free_plan_buffers(tc_plan *p) {
    if (p->upload_event) {
        (void)hipEventSynchronize((hipEvent_t)p->upload_event);
        (void)hipEventDestroy((hipEvent_t)p->upload_event);
        p->upload_event = nullptr;
    }
    if (p->dev) (void)hipFree(p->dev);
    p->dev = nullptr;
    p->dev_cap = 0;
    if (p->host) {
        if (p->host_pinned) (void)hipHostFree(p->host); else std::free(p->host);
    }
    p->host = nullptr;
    p->host_cap = p->host_n = 0;
}

// ------------------------------------------------------------------------------------
// Launchers
// ------------------------------------------------------------------------------------
int launch_kv_append(const tc_plan *p, const tc_kv_pool *pool, const void *k_new, const void *v_new, bool only_prefill, void *stream) {
    const int n = only_prefill ? p->n_append_prefill : p->n_append;
    if (n == 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((unsigned)n, (unsigned)p->Hkv);  // Hkv <= 1024 is checked when the plan is built
    if (p->D == 128)
        kv_append_kernel<128><<<grid, 512, 0, st>>>((uint16_t *)pool->k_pool, (uint16_t *)pool->v_pool, (const uint16_t *)k_new,
                                                   (const uint16_t *)v_new, p->dev + p->off_append, p->Hkv);
    else
        kv_append_kernel<64><<<grid, 256, 0, st>>>((uint16_t *)pool->k_pool, (uint16_t *)pool->v_pool, (const uint16_t *)k_new,
                                                  (const uint16_t *)v_new, p->dev + p->off_append, p->Hkv);
    return (int)hipGetLastError();
}

int launch_kv_gather(const tc_plan *p, const tc_kv_pool *pool, int seq, void *k_out, void *v_out, void *stream) {
    const int kv_len = p->ctx_len[seq] + (p->q_start[seq + 1] - p->q_start[seq]);
    const int64_t total = (int64_t)kv_len * p->Hkv * (p->D / 8);
    const unsigned blocks = (unsigned)((total + 255) / 256);
    hipStream_t st = (hipStream_t)stream;
    const int32_t *pages = p->dev + p->off_pages + p->page_off[seq];
    if (p->D == 128)
        kv_gather_kernel<128><<<blocks, 256, 0, st>>>((const uint16_t *)pool->k_pool, (const uint16_t *)pool->v_pool, pages, kv_len,
                                                     p->Hkv, (uint16_t *)k_out, (uint16_t *)v_out);
    else
        kv_gather_kernel<64><<<blocks, 256, 0, st>>>((const uint16_t *)pool->k_pool, (const uint16_t *)pool->v_pool, pages, kv_len,
                                                    p->Hkv, (uint16_t *)k_out, (uint16_t *)v_out);
    return (int)hipGetLastError();
}

int launch_kv_migrate(const tc_plan *p, bool import, int page0, int n_pages, int num_layers, void *const *k_pools,
                      void *const *v_pools, void *buffer, void *stream) {
    if (n_pages == 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    const int block_pieces = p->Hkv * p->D * 2;  // 16-byte pieces of one block of one pool
    const int64_t layer_stride = (int64_t)n_pages * 2 * block_pieces * 8;  // buffer elements per layer
    const int32_t *pages = p->dev + p->off_pages + page0, *valid = p->dev + p->off_valid + page0;
    for (int l0 = 0; l0 < num_layers; l0 += kMigrateLayers) {
        const int nl = std::min(kMigrateLayers, num_layers - l0);
        MigratePools mp;
        for (int l = 0; l < kMigrateLayers; l++) {
            mp.k[l] = (uint16_t *)k_pools[l0 + std::min(l, nl - 1)];
            mp.v[l] = (uint16_t *)v_pools[l0 + std::min(l, nl - 1)];
        }
        uint16_t *buf = (uint16_t *)buffer + (int64_t)l0 * layer_stride;
        const dim3 grid((unsigned)n_pages, (unsigned)nl);
        if (import)
            kv_migrate_kernel<true><<<grid, 256, 0, st>>>(mp, pages, valid, buf, layer_stride, block_pieces);
        else
            kv_migrate_kernel<false><<<grid, 256, 0, st>>>(mp, pages, valid, buf, layer_stride, block_pieces);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return (int)e;
    }
    return 0;
}

// More than 64 KiB of dynamic LDS needs an opt-in per kernel function and per device; remembered per
// instantiation and device (setting it twice is harmless, so racing first calls need no lock).
template <int D, class E>
static int allow_prefill_lds(int device) {
    static std::atomic<bool> done[kMaxDevices];
    const bool known = device >= 0 && device < kMaxDevices;
    if (known && done[device].load(std::memory_order_acquire)) return 0;
    hipError_t e = hipFuncSetAttribute((const void *)mixed_attention_kernel<D, E, kMixedWaves>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, PrefillCfg<D>::kLdsBytes);
    if (e != hipSuccess) return (int)e;
    if (known) done[device].store(true, std::memory_order_release);
    return 0;
}

template <int D, class E>
static int launch_attention_d(const tc_plan *p, const AttnArgs &A, int launches, hipStream_t st) {
    int grid = (launches & (kLaunchAttention | kLaunchFused)) ? p->grid_blocks() : 0;
    // A batch of decodes whose rows this launch stores: workgroups at the back of the grid do it (four (row, KV head,
    // 8-element piece) units per thread).  A batch with a prefill chunk never gets here with k_new set (see launch_attention).
    int n_front = 0;
    if (grid > 0 && A.k_new && p->n_pieces == 0) {
        const int64_t units = (int64_t)p->n_append * p->Hkv * (D / 8);
        n_front = (int)((units + kDecodeWaves * 64 * 4 - 1) / (kDecodeWaves * 64 * 4));
        grid += n_front;
    }
    const AttnScalars sc = {A.n_prefill, A.n_decode, A.Hq, A.Hkv, A.G, A.fused, A.queue, p->n_partials, n_front, p->n_append, A.scale_log2};
    const int32_t *append = p->dev + p->off_append;
    if (grid > 0 && p->n_pieces > 0) {
        const int lds = PrefillCfg<D>::kLdsBytes;  // the decode workgroups of the launch need less, for any G
        static_assert(decode_team_lds_bytes(kMixedWaves, 16, D) <= (size_t)PrefillCfg<D>::kLdsBytes, "team buffers must fit the prefill tiles' LDS");
        if (int err = allow_prefill_lds<D, E>(p->device)) return err;
        mixed_attention_kernel<D, E, kMixedWaves><<<grid, kMixedWaves * 64, lds, st>>>(
            A.k_pool, A.v_pool, A.q, A.k_new, A.v_new, A.out, A.pages, A.prefill, A.pieces, A.wg_first, A.decode, A.merge, append,
            A.counters, A.ws_o, sc);
    } else if (grid > 0) {
        mixed_attention_kernel<D, E, kDecodeWaves><<<grid, kDecodeWaves * 64, decode_team_lds_bytes(kDecodeWaves, p->G, D), st>>>(
            A.k_pool, A.v_pool, A.q, A.k_new, A.v_new, A.out, A.pages, A.prefill, A.pieces, A.wg_first, A.decode, A.merge, append,
            A.counters, A.ws_o, sc);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
    if ((launches & kLaunchMerge) && p->n_merge_prefill > 0) {
        prefill_merge_kernel<D, E><<<p->n_merge_prefill, kMixedWaves * 64, 0, st>>>(p->dev + p->off_merge, p->dev + p->off_prefill, A.ws_pieces,
                                                                                    A.out, A.Hq, A.G);
        e = hipGetLastError();
        if (e != hipSuccess) return (int)e;
    }
    if ((launches & kLaunchMerge) && p->n_merge > p->n_merge_prefill)
        split_merge_kernel<D, E><<<p->n_merge - p->n_merge_prefill, 256, 0, st>>>(p->dev + p->off_merge + (size_t)p->n_merge_prefill * kItemInts,
                                                                                 A.ws_o, A.ws_ml, A.out, A.Hq, A.G);
    return (int)hipGetLastError();
}

int launch_attention(const tc_plan *p, const tc_kv_pool *pool, const void *q, const void *k_new, const void *v_new, void *out,
                     float scale, void *workspace, int launches, void *stream) {
    AttnArgs A;
    A.k_pool = (uint16_t *)pool->k_pool;
    A.v_pool = (uint16_t *)pool->v_pool;
    A.q = (const uint16_t *)q;
    // only a batch of decodes has its rows stored by the attention launch itself
    A.k_new = p->n_pieces == 0 ? (const uint16_t *)k_new : nullptr;
    A.v_new = p->n_pieces == 0 ? (const uint16_t *)v_new : nullptr;
    A.out = (uint16_t *)out;
    A.pages = p->dev + p->off_pages;
    A.prefill = p->dev + p->off_prefill;
    A.pieces = p->dev + p->off_pieces;
    A.wg_first = p->dev + p->off_wg;
    A.decode = p->dev + p->off_decode;
    A.merge = p->dev + p->off_merge;
    A.counters = p->dev + p->off_counters;
    A.ws_o = (float *)workspace;
    A.ws_ml = A.ws_o ? A.ws_o + (size_t)p->n_partials * p->G * p->D : nullptr;
    A.ws_pieces = A.ws_o ? A.ws_ml + (size_t)p->n_partials * p->G * 2 : nullptr;
    A.n_prefill = p->n_prefill_wg;
    A.n_decode = p->n_decode;
    A.Hq = p->Hq;
    A.Hkv = p->Hkv;
    A.G = p->G;
    A.fused = (launches & kLaunchFused) ? 1 : 0;
    A.queue = p->queue_counter;
    A.scale_log2 = scale * 1.4426950408889634f;
    hipStream_t st = (hipStream_t)stream;
    if (p->dtype == TC_FP16) return p->D == 128 ? launch_attention_d<128, Fp16>(p, A, launches, st) : launch_attention_d<64, Fp16>(p, A, launches, st);
    return p->D == 128 ? launch_attention_d<128, Bf16>(p, A, launches, st) : launch_attention_d<64, Bf16>(p, A, launches, st);
}

// ------------------------------------------------------------------------------------
// Static scratch: a workspace for callers that cannot allocate
// ------------------------------------------------------------------------------------
// Partial results of split KV ranges for tc_mixed_attention_static.  Every GPU the library runs on holds
// its own copy of the array, at its own address, until the process ends.  Host code never uses the
// array's name as an address: the device address is asked for once per device and kept.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

int static_scratch(int device, void **ptr, size_t *bytes) {
    static std::atomic<void *> address[kMaxDevices];
    *bytes = kStaticScratchBytes;
    *ptr = nullptr;
    if (device < 0 || device >= kMaxDevices) return (int)hipErrorInvalidDevice;
    void *a = address[device].load(std::memory_order_acquire);
    if (!a) {
        int current = -1;
        hipError_t e = hipGetDevice(&current);
        if (e != hipSuccess) return (int)e;
        if (current != device) return (int)hipErrorInvalidDevice;  // the address is that of the current device's copy
        e = hipGetSymbolAddress(&a, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return (int)e;
        if (!a) return (int)hipErrorInvalidSymbol;
        address[device].store(a, std::memory_order_release);
    }
    *ptr = a;
    return 0;
}

}  // namespace tc

#ifdef TC_WG_TRACE
// Tracing build only: copy the first n int64 of the workgroup trace of the latest attention launch to HOST memory.
extern "C" int tc_debug_wg_trace(long long *dst, int n) {
    (void)hipDeviceSynchronize();
    return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(tc::g_wg_trace), (size_t)n * sizeof(long long));
}
#endif
