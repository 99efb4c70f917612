// Fused W-way gradient reduction + scale + momentum-SGD update for gfx950.
//
// This translation unit is compiled once per (gradient dtype, W) pair, selected
// by -DKV_TU_F16={0,1} and -DKV_TU_W={0,2,4,8,16,32} (0 = W known only at run
// time), and exports one launcher, kv_launch_fused_f<F16>_w<W>.
//
// The path is a pure streaming pass: per parameter element it reads W gradient
// values once, reads w and m, and writes w' and m'.  There is no reuse, so there
// is no LDS staging and no MFMA; what matters is that every lane issues
// independent loads (N = 1, 2 or 4 consecutive elements per lane and rank; all W ranks, and `U`
// such vectors per rank, are in flight before the first add) and that a wavefront's 64 lanes cover
// contiguous memory per load instruction.  On MI355X the memory system is fastest with roughly
// 80 KB in flight per compute unit in as many small requests as possible: for 8 fp32 ranks that
// is N = 1, U = 1 (40 bytes per lane, workgroups of 256 elements), not 16-byte vectors.
//
// Arithmetic contract (must match bit for bit what the header of the C ABI
// states): each element is owned by one lane for all W ranks, the ranks are
// folded in a fixed order, every operation is a separate IEEE binary32 operation.
// The file must be compiled with -ffp-contract=off.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kv_device.hpp"
#include "kv_kernels.hpp"

#ifndef KV_TU_F16
#error "KV_TU_F16 must be defined"
#endif
#ifndef KV_TU_W
#error "KV_TU_W must be defined"
#endif

// Kernel for a W known only at run time: gradient bytes per lane whose loads are issued back to back
// (one batch of ranks); the batch is this many bytes divided by the size of a lane's vector.
#ifndef KV_RUNTIME_W_BYTES
#define KV_RUNTIME_W_BYTES 128
#endif

namespace {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

// N consecutive fp32 / fp16 values as one register-resident vector (a plain scalar for N = 1).
template <int N> struct FVec;
template <> struct FVec<1> { using type = float; };
template <> struct FVec<2> { using type = f32x2; };
template <> struct FVec<4> { using type = f32x4; };
template <int N> struct HVec;
template <> struct HVec<1> { using type = _Float16; };
template <> struct HVec<2> { using type = f16x2; };
template <> struct HVec<4> { using type = f16x4; };

template <int N, typename V>
__device__ __forceinline__ float lane_get(const V& v, int i) {
    if constexpr (N == 1) return (float)v;
    else return (float)v[i];
}
template <int N>
__device__ __forceinline__ typename FVec<N>::type pack_f32(const float (&a)[N]) {
    if constexpr (N == 1) return a[0];
    else {
        typename FVec<N>::type v;
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = a[i];
        return v;
    }
}
template <int N>
__device__ __forceinline__ typename HVec<N>::type pack_f16(const float (&a)[N]) {       // round to nearest even
    if constexpr (N == 1) return (_Float16)a[0];
    else {
        typename HVec<N>::type v;
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = (_Float16)a[i];
        return v;
    }
}

// Gradient vector of one lane: N consecutive elements.  Whatever the gradient dtype, a lane then
// owns exactly one N-element vector of w and of m, so that every load and store of the fp32 state
// of a wavefront covers whole cache lines.  (With 8 halves per lane and two state vectors the
// state accesses touched every line half, twice; measured 9 % slower on ResNet-50 W=32.)
template <bool F16, int N> struct Grad {
    using elem = float;
    using vec = typename FVec<N>::type;
};
template <int N> struct Grad<true, N> {
    using elem = _Float16;
    using vec = typename HVec<N>::type;
};
// Widening is exact: every binary16 value is a binary32 value.
template <int N, typename V>
__device__ __forceinline__ void widen(const V& v, float (&o)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i) o[i] = lane_get<N>(v, i);
}

// Cache-policy mask of a kernel instantiation:
//   bit 0       gradient loads carry the non-temporal hint
//   bit 1       loads of w and m carry it (measured slower; not instantiated)
//   bits 2..3   stores of w', m' (and s): 0 = plain, 4 = non-temporal, 8 = agent scope (write through L2),
//               12 = both
template <bool NT, typename T>
__device__ __forceinline__ T load_grad(const T* p) {
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT, int N>
__device__ __forceinline__ typename FVec<N>::type load_state(const float* p) {
    using V = typename FVec<N>::type;
    if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const V*>(p));
    else return *reinterpret_cast<const V*>(p);
}
// Stores N floats at element `k` of the uniform base pointer `base`.  Policies 8 and 12 use a raw
// buffer store, whose cache-policy operand can carry the sc1 bit (write through L2 to memory
// at once instead of leaving a dirty line in L2); the buffer descriptor spans exactly the
// bytes handed in, so an out-of-range lane could not write.  0x00020000 is word 3 of a raw
// (untyped, 32-bit data format) buffer descriptor on gfx9-family targets.
template <int POL, int N>
__device__ __forceinline__ void store_state(float* base, int k, unsigned span_bytes, const typename FVec<N>::type& v) {
    using V = typename FVec<N>::type;
    if constexpr (POL == 4) {
        __builtin_nontemporal_store(v, reinterpret_cast<V*>(base + k));
    } else if constexpr (POL == 8 || POL == 12) {
        typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
        typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(base, 0, span_bytes, 0x00020000);
        constexpr int aux = POL == 12 ? /*sc1 + nt*/ 18 : /*sc1*/ 16;
        if constexpr (N == 4) __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), rsrc, k * 4, 0, aux);
        else if constexpr (N == 2) __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, v), rsrc, k * 4, 0, aux);
        else __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), rsrc, k * 4, 0, aux);
    } else {
        *reinterpret_cast<V*>(base + k) = v;
    }
}

// Rank-order left fold: s = g_0; s = s + g_r.  The first term is taken as is.
template <int NV> struct FoldSeq {
    float acc[NV];
    unsigned count = 0;
    __device__ __forceinline__ void push(const float (&v)[NV]) {
        if (count == 0) {
#pragma unroll
            for (int i = 0; i < NV; ++i) acc[i] = v[i];
        } else {
#pragma unroll
            for (int i = 0; i < NV; ++i) acc[i] = acc[i] + v[i];
        }
        ++count;
    }
    // a rank that is known not to be the first one
    __device__ __forceinline__ void push_next(const float (&v)[NV]) {
#pragma unroll
        for (int i = 0; i < NV; ++i) acc[i] = acc[i] + v[i];
        ++count;
    }
    __device__ __forceinline__ void finish(float (&o)[NV]) const {
#pragma unroll
        for (int i = 0; i < NV; ++i) o[i] = acc[i];
    }
};

// Balanced tree in rank order, evaluated as a stream with a binary-counter stack:
// level l holds the sum of a complete block of 2^l consecutive ranks.  After n
// pushes the occupied levels are the set bits of n, leftmost block highest; the
// final merge runs from the lowest level up with the earlier block on the left.
// This is sum(lo,n) = sum(lo,h) + sum(lo+h,n-h), h = largest power of two < n.
template <int NV> struct FoldPair {
    static constexpr int L = 9;               // up to 2^8 = KV_MAX_W ranks
    float st[L][NV];
    unsigned count = 0;
    __device__ __forceinline__ void push(const float (&v)[NV]) {
        float cur[NV];
#pragma unroll
        for (int i = 0; i < NV; ++i) cur[i] = v[i];
        unsigned c = count;
        bool placed = false;
#pragma unroll
        for (int l = 0; l < L; ++l) {
            if (!placed) {
                if (c & 1u) {
#pragma unroll
                    for (int i = 0; i < NV; ++i) cur[i] = st[l][i] + cur[i];
                    c >>= 1;
                } else {
#pragma unroll
                    for (int i = 0; i < NV; ++i) st[l][i] = cur[i];
                    placed = true;
                }
            }
        }
        ++count;
    }
    __device__ __forceinline__ void push_next(const float (&v)[NV]) { push(v); }
    __device__ __forceinline__ void finish(float (&o)[NV]) const {
        bool have = false;
#pragma unroll
        for (int l = 0; l < L; ++l) {
            if ((count >> l) & 1u) {
                if (!have) {
#pragma unroll
                    for (int i = 0; i < NV; ++i) o[i] = st[l][i];
                    have = true;
                } else {
#pragma unroll
                    for (int i = 0; i < NV; ++i) o[i] = st[l][i] + o[i];
                }
            }
        }
    }
};

template <int NV, bool PAIRWISE> struct FoldSel { using type = FoldSeq<NV>; };
template <int NV> struct FoldSel<NV, true> { using type = FoldPair<NV>; };

// The tile table and the gradient-pointer table are written by the host before the
// launch and never by a kernel, so they are read through the constant address
// space: uniform addresses become scalar loads (s_load) instead of vector loads plus
// readfirstlane.  Gradient buffers are read through the global address space
// (global_load, not flat_load).
#define KV_CONST __attribute__((address_space(4)))
#define KV_GLOBAL __attribute__((address_space(1)))

// Placed after the gradient loads of a batch: the instruction scheduler may move nothing across it.  Without it
// the arithmetic on w and m -- which comes later in program order but depends only on loads issued earlier --
// has been seen hoisted in front of the gradient loads together with its wait for w and m, which puts two memory
// round trips one after the other (ResNet-50, 8 fp32 ranks: 169 -> 177 us).
__device__ __forceinline__ void loads_issued() { __builtin_amdgcn_sched_barrier(0); }

// Ranks r0 .. r0 + RB - 1 (GUARDED: those below W) of one lane's vector: all loads first, then the fold.
template <bool F16, int N, int RB, bool GUARDED, bool NT, typename Fold>
__device__ __forceinline__ void fold_batch(Fold& f, const uint64_t KV_CONST* gp, int r0, int W, int64_t boff) {
    using V = typename Grad<F16, N>::vec;
    V g[RB];
#pragma unroll
    for (int j = 0; j < RB; ++j)
        if (!GUARDED || r0 + j < W) g[j] = load_grad<NT>((const V KV_GLOBAL*)(gp[r0 + j] + (uint64_t)boff));
    loads_issued();
#pragma unroll
    for (int j = 0; j < RB; ++j) {
        if (!GUARDED || r0 + j < W) {
            float t[N];
            widen<N>(g[j], t);
            if (j == 0) f.push(t);          // only a batch's first rank can be the first rank of all
            else f.push_next(t);
        }
    }
}

// The last W - r0 < RS ranks (RS = 8 or 4) as pieces of 4, 2 and 1 ranks: the loads of all pieces are issued
// before the first fold, behind three uniform branches.  (One guarded load per rank, each behind its own
// branch, came out as one memory round trip per rank.)
template <bool F16, int N, int RS, bool NT, typename Fold>
__device__ __forceinline__ void fold_tail(Fold& f, const uint64_t KV_CONST* gp, int r0, int W, int64_t boff) {
    using V = typename Grad<F16, N>::vec;
    const int rem = W - r0;
    const bool h4 = RS > 4 && (rem & 4) != 0, h2 = (rem & 2) != 0, h1 = (rem & 1) != 0;
    const int r4 = r0, r2 = r4 + (h4 ? 4 : 0), r1 = r2 + (h2 ? 2 : 0);
    V g4[4], g2[2], g1;
    if (h4) {
#pragma unroll
        for (int j = 0; j < 4; ++j) g4[j] = load_grad<NT>((const V KV_GLOBAL*)(gp[r4 + j] + (uint64_t)boff));
    }
    if (h2) {
#pragma unroll
        for (int j = 0; j < 2; ++j) g2[j] = load_grad<NT>((const V KV_GLOBAL*)(gp[r2 + j] + (uint64_t)boff));
    }
    if (h1) g1 = load_grad<NT>((const V KV_GLOBAL*)(gp[r1] + (uint64_t)boff));
    loads_issued();
    float t[N];
    if (h4) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            widen<N>(g4[j], t);
            if (j == 0) f.push(t);
            else f.push_next(t);
        }
    }
    if (h2) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            widen<N>(g2[j], t);
            if (j == 0) f.push(t);
            else f.push_next(t);
        }
    }
    if (h1) {
        widen<N>(g1, t);
        f.push(t);
    }
}

// Sum over ranks of the gradient vector (N values) that starts `boff` bytes into every rank's copy of the key.
template <bool F16, int N, int WT, bool PAIRWISE, bool NT>
__device__ __forceinline__ void reduce_vec(const uint64_t KV_CONST* gp, int W, int64_t boff, float (&s)[N]) {
    using V = typename Grad<F16, N>::vec;
    typename FoldSel<N, PAIRWISE>::type f;
    if constexpr (WT > 0) {
        constexpr int CH = WT > 16 ? 16 : WT;      // ranks whose loads are issued back to back
#pragma unroll
        for (int r0 = 0; r0 < WT; r0 += CH) {
            V g[CH];
#pragma unroll
            for (int j = 0; j < CH; ++j) g[j] = load_grad<NT>((const V KV_GLOBAL*)(gp[r0 + j] + (uint64_t)boff));
            loads_issued();
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                float t[N];
                widen<N>(g[j], t);
                f.push(t);
            }
        }
    } else {
        // W known only at run time: whole large batches (KV_RUNTIME_W_BYTES of gradients per lane in flight), at
        // most one batch of half that size, then whole small batches, then the tail; always in rank order.
        constexpr int RL0 = KV_RUNTIME_W_BYTES / (int)sizeof(V);
        constexpr int RL = RL0 < 8 ? 8 : RL0 > 32 ? 32 : RL0;
        constexpr int RM = RL / 2;                   // 16 .. 31 ranks of 4-byte vectors: one batch of 16 first
        constexpr int RS = RL > 8 ? 8 : 4;
        int r0 = 0;
        for (; r0 + RL <= W; r0 += RL) fold_batch<F16, N, RL, false, NT>(f, gp, r0, W, boff);
        if constexpr (RM > RS) {
            if (r0 + RM <= W) {
                fold_batch<F16, N, RM, false, NT>(f, gp, r0, W, boff);
                r0 += RM;
            }
        }
        // fewer than 2 RS ranks are left here (RL is 2 RS or 4 RS, and RM = 2 RS in the latter case)
        static_assert(RL == 2 * RS || (RL == 4 * RS && RM == 2 * RS), "batch tiers");
        if (r0 + RS <= W) {
            fold_batch<F16, N, RS, false, NT>(f, gp, r0, W, boff);
            r0 += RS;
        }
        if (r0 < W) fold_tail<F16, N, RS, NT>(f, gp, r0, W, boff);
    }
    f.finish(s);
}

// Same for the single element `e` of the key (ragged tails and gradient buffers
// that are not 16-byte aligned).
template <bool F16, int WT, bool PAIRWISE>
__device__ __forceinline__ float reduce_one(const uint64_t KV_CONST* gp, int W, int64_t e) {
    using E = typename Grad<F16, 1>::elem;
    typename FoldSel<1, PAIRWISE>::type f;
    const int n = WT > 0 ? WT : W;
    for (int r = 0; r < n; ++r) {
        float t[1] = {(float)((const E KV_GLOBAL*)gp[r])[e]};
        f.push(t);
    }
    float o[1];
    f.finish(o);
    return o[0];
}

// eq. (1) extended by momentum and weight decay; one rounding per operation.
__device__ __forceinline__ void sgd_update(float s, float w, float m, float rescale, float lr, float mu, float wd,
                                           float& w_new, float& m_new) {
    const float ghat = rescale * s;
    const float wdw = wd * w;
    const float t = ghat + wdw;
    const float mm = mu * m;
    const float lt = lr * t;
    const float dw = mm - lt;
    m_new = dw;
    w_new = w + dw;
}

// Third phase of the paper's collective (every GPU receives the final result): the updated
// weights also go to `n` replica buffers of the key, as fp32 or rounded to nearest-even fp16, in
// the same pass.  row == nullptr or a null first pointer: the key has no replicas.  The replicas are
// pure output streams: their stores carry the non-temporal hint, so that (with 8 fp32 replicas) 818 MB
// of them per step do not push w and m out of the memory-side cache (0.377 -> 0.299 ms on ResNet-50).
struct Bcast {
    const uint64_t KV_CONST* row;
    int n;
    int f16;
};

template <int N>
__device__ __forceinline__ void bcast_vec(const Bcast& b, int64_t e, const float (&wn)[N]) {
    if (b.n == 0) return;
    if (b.f16) {
        const typename HVec<N>::type h = pack_f16<N>(wn);
        for (int r = 0; r < b.n; ++r)
            __builtin_nontemporal_store(h, (typename HVec<N>::type KV_GLOBAL*)(b.row[r] + (uint64_t)e * 2u));
    } else {
        const typename FVec<N>::type v = pack_f32<N>(wn);
        for (int r = 0; r < b.n; ++r)
            __builtin_nontemporal_store(v, (typename FVec<N>::type KV_GLOBAL*)(b.row[r] + (uint64_t)e * 4u));
    }
}

__device__ __forceinline__ void bcast1(const Bcast& b, int64_t e, float wn) {
    if (b.n == 0) return;
    if (b.f16) {
        for (int r = 0; r < b.n; ++r) __builtin_nontemporal_store((_Float16)wn, (_Float16 KV_GLOBAL*)b.row[r] + e);
    } else {
        for (int r = 0; r < b.n; ++r) __builtin_nontemporal_store(wn, (float KV_GLOBAL*)b.row[r] + e);
    }
}

// Element `k` of the tile: e = element index inside the key, wp/mp/sp point at the tile start.
template <bool F16, int WT, bool PAIRWISE, bool KEEP>
__device__ __forceinline__ void scalar_element(const uint64_t KV_CONST* gp, int W, int64_t e, int k,
                                               float* __restrict__ wp, float* __restrict__ mp, float* __restrict__ sp,
                                               const Bcast& bc, const KvLaunchArgs& a) {
    const float s = reduce_one<F16, WT, PAIRWISE>(gp, W, e);
    float wn, mn;
    sgd_update(s, wp[k], mp[k], a.rescale, a.lr, a.momentum, a.wd, wn, mn);
    if constexpr (KEEP) sp[k] = s;
    mp[k] = mn;
    wp[k] = wn;
    bcast1(bc, e, wn);
}

// Updates the N elements k..k+N-1 of the tile whose arenas start at wp / mp / sp.
template <bool KEEP, int NTS, int N>
__device__ __forceinline__ void update_store(const float (&s)[N], const typename FVec<N>::type& wv,
                                             const typename FVec<N>::type& mv, float* wp, float* mp, float* sp, int k,
                                             unsigned span_bytes, const Bcast& bc, int64_t e, const KvLaunchArgs& a) {
    float wn[N], mn[N];
#pragma unroll
    for (int c = 0; c < N; ++c)
        sgd_update(s[c], lane_get<N>(wv, c), lane_get<N>(mv, c), a.rescale, a.lr, a.momentum, a.wd, wn[c], mn[c]);
    // the raw sums are an output stream that no later launch reads: write-through and non-temporal
    // whatever the policy of w' and m', so that they do not push w and m out of the memory-side cache
    if constexpr (KEEP) store_state<12, N>(sp, k, span_bytes, pack_f32<N>(s));
    store_state<NTS, N>(mp, k, span_bytes, pack_f32<N>(mn));
    store_state<NTS, N>(wp, k, span_bytes, pack_f32<N>(wn));
    bcast_vec<N>(bc, e, wn);
}

template <bool F16, int N, int WT, bool PAIRWISE, bool KEEP, int U, int NTM>
__global__ void __launch_bounds__(KV_THREADS) kv_fused(const KvLaunchArgs a) {
    using E = typename Grad<F16, N>::elem;
    using FV = typename FVec<N>::type;
    constexpr int TILE = KV_THREADS * N * U;
    constexpr bool NT = (NTM & 1) != 0;      // gradient loads
    constexpr bool NTL = (NTM & 2) != 0;     // w, m loads
    constexpr int NTS = NTM & 12;            // store policy of w', m', s
    const int W = WT > 0 ? WT : a.W;
    const int tid = threadIdx.x;

    // a KvTile as four 64-bit words: {seg | count << 32, arena_off, seg_off, reserved}
    static_assert(sizeof(KvTile) == 32, "tile layout");
    const int64_t KV_CONST* tiles = (const int64_t KV_CONST*)a.tiles + a.tile_lo * 4;
    const uint64_t KV_CONST* table = (const uint64_t KV_CONST*)a.gptrs;

    // The hardware deals consecutive workgroup ids round-robin to the 8 XCDs.  xcd_remap = G > 0 gives
    // every XCD blocks of G consecutive tiles (rows of 8 G tiles, block x of a row to XCD x; G = an
    // eighth of the launch: eight contiguous ranges); 0 leaves the tiles dealt one by one.  All in
    // 32-bit unsigned arithmetic (the host keeps a launch below 2^31 tiles), with shifts when G is
    // a power of two: this runs once per workgroup, and a workgroup may be as small as 256 elements.
    const uint32_t ntiles = (uint32_t)(a.tile_hi - a.tile_lo);
    const uint32_t blk = (uint32_t)a.xcd_remap;
    const uint32_t row_len = 8u * blk;
    const int blk_shift = a.xcd_shift;                       // log2(G), or -1 if G is not a power of two
    const uint32_t span = a.xcd_span;                        // ntiles rounded up to whole rows (ntiles if G = 0)

    for (uint32_t i = blockIdx.x; i < span; i += gridDim.x) {
        uint32_t t = i;
        if (blk) {
            uint32_t row_start, within;
            if (blk_shift >= 0) {
                within = i & (row_len - 1u);
                row_start = i - within;
                t = row_start + ((within & 7u) << blk_shift) + (within >> 3);
            } else {
                row_start = i / row_len * row_len;
                within = i - row_start;
                t = row_start + (within & 7u) * blk + (within >> 3);
            }
            if (t >= ntiles) continue;
        }
        struct { int32_t seg, count; int64_t arena_off, seg_off; } td;
        {
            // the whole 32-byte descriptor in one scalar load (loaded word by word, the word that is needed last
            // has been seen fetched by a later, dependent load)
            typedef int64_t i64x4 __attribute__((ext_vector_type(4)));
            const i64x4 d = *(const i64x4 KV_CONST*)(tiles + (int64_t)t * 4);
            td.seg = (int32_t)(d[0] & 0xFFFFFFFF);
            td.count = (int32_t)(d[0] >> 32);
            td.arena_off = d[1];
            td.seg_off = d[2];
        }
        float* __restrict__ wp = a.w + td.arena_off;
        float* __restrict__ mp = a.m + td.arena_off;
        float* __restrict__ sp = KEEP ? a.s + td.arena_off : nullptr;
        const uint64_t KV_CONST* gp = table + (int64_t)td.seg * W;
        const bool full = td.count == TILE;
        const unsigned span_bytes = (unsigned)td.count * 4u;      // bytes of this tile in each arena

        // A full tile lies wholly inside the arena, so its w and m vectors can be requested
        // before the gradient pointers have arrived (they are dropped in the rare case that
        // the gradient buffers turn out not to be aligned to one vector).
        FV wv[U], mv[U];
        if (full) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int k = (tid + u * KV_THREADS) * N;
                wv[u] = load_state<NTL, N>(wp + k);
                mv[u] = load_state<NTL, N>(mp + k);
            }
        }

        // The vector path needs every gradient pointer aligned to one gradient vector (N elements)
        // and every replica pointer to one replica vector.
        // The host hands over the OR of all gradient pointers of the launch; only if some buffer of the
        // launch is misaligned for this lane width does a tile look at its own key's pointers (W dependent
        // scalar loads when W is known only at run time).
        uint64_t bits = a.grad_align;
        if (bits & (uint64_t)(N * sizeof(E) - 1)) {
            bits = 0;
            for (int r = 0; r < W; ++r) bits |= gp[r];
        }
        bool vec_ok = (bits & (uint64_t)(N * sizeof(E) - 1)) == 0;

        Bcast bc{nullptr, 0, a.bcast_f16};
        if (a.bcast_n > 0) {
            const uint64_t KV_CONST* row = (const uint64_t KV_CONST*)a.bcast + (int64_t)td.seg * a.bcast_n;
            if (row[0] != 0) {
                bc.row = row;
                bc.n = a.bcast_n;
                uint64_t rbits = 0;
                for (int r = 0; r < a.bcast_n; ++r) rbits |= row[r];
                vec_ok = vec_ok && (rbits & (uint64_t)(N * (a.bcast_f16 ? 2 : 4) - 1)) == 0;
            }
        }

        if (vec_ok && full) {
            // every gradient load of every unrolled vector is issued before the first store
            float s[U][N];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t e = td.seg_off + (int64_t)(tid + u * KV_THREADS) * N;
                reduce_vec<F16, N, WT, PAIRWISE, NT>(gp, W, e * (int64_t)sizeof(E), s[u]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int k = (tid + u * KV_THREADS) * N;
                update_store<KEEP, NTS, N>(s[u], wv[u], mv[u], wp, mp, sp, k, span_bytes, bc, td.seg_off + k, a);
            }
        } else if (vec_ok) {
            // ragged tile: whole vectors first, then at most N-1 single elements
            const int nvec = td.count / N;
            for (int v = tid; v < nvec; v += KV_THREADS) {
                const int k = v * N;
                float s[N];
                reduce_vec<F16, N, WT, PAIRWISE, NT>(gp, W, (td.seg_off + k) * (int64_t)sizeof(E), s);
                const FV w1 = load_state<NTL, N>(wp + k);
                const FV m1 = load_state<NTL, N>(mp + k);
                update_store<KEEP, NTS, N>(s, w1, m1, wp, mp, sp, k, span_bytes, bc, td.seg_off + k, a);
            }
            const int rem = td.count - nvec * N;
            if (tid < rem) {
                const int k = nvec * N + tid;
                scalar_element<F16, WT, PAIRWISE, KEEP>(gp, W, td.seg_off + k, k, wp, mp, sp, bc, a);
            }
        } else {
            for (int k = tid; k < td.count; k += KV_THREADS)
                scalar_element<F16, WT, PAIRWISE, KEEP>(gp, W, td.seg_off + k, k, wp, mp, sp, bc, a);
        }
    }
}

template <bool F16, int N, int WT, bool PAIRWISE, bool KEEP, int U, int NTM>
hipError_t launch_one(const KvLaunchArgs& a, unsigned grid, hipStream_t st) {
    hipLaunchKernelGGL((kv_fused<F16, N, WT, PAIRWISE, KEEP, U, NTM>), dim3(grid), dim3(KV_THREADS), a.lds_pad, st, a);
    return hipGetLastError();
}

template <bool F16, int N, int WT, bool PAIRWISE, bool KEEP, int U>
hipError_t pick_nt(const KvKernelSel& s, const KvLaunchArgs& a, unsigned grid, hipStream_t st) {
    switch (s.nontemporal) {
        case 0: return launch_one<F16, N, WT, PAIRWISE, KEEP, U, 0>(a, grid, st);
        case 1: return launch_one<F16, N, WT, PAIRWISE, KEEP, U, 1>(a, grid, st);
        case 5: return launch_one<F16, N, WT, PAIRWISE, KEEP, U, 5>(a, grid, st);
        case 9: return launch_one<F16, N, WT, PAIRWISE, KEEP, U, 9>(a, grid, st);
        case 13: return launch_one<F16, N, WT, PAIRWISE, KEEP, U, 13>(a, grid, st);
        default: return hipErrorInvalidValue;
    }
}

// (elements per lane, vectors per lane): 4 x {1, 2, 4}, 2 x {1, 2}, 1 x {1, 2, 4}
template <bool F16, int WT, bool PAIRWISE, bool KEEP>
hipError_t pick_shape(const KvKernelSel& s, const KvLaunchArgs& a, unsigned grid, hipStream_t st) {
    switch (s.lane_elems * 8 + s.unroll) {
        case 4 * 8 + 1: return pick_nt<F16, 4, WT, PAIRWISE, KEEP, 1>(s, a, grid, st);
        case 4 * 8 + 2: return pick_nt<F16, 4, WT, PAIRWISE, KEEP, 2>(s, a, grid, st);
        case 4 * 8 + 4: return pick_nt<F16, 4, WT, PAIRWISE, KEEP, 4>(s, a, grid, st);
        case 2 * 8 + 1: return pick_nt<F16, 2, WT, PAIRWISE, KEEP, 1>(s, a, grid, st);
        case 2 * 8 + 2: return pick_nt<F16, 2, WT, PAIRWISE, KEEP, 2>(s, a, grid, st);
        case 1 * 8 + 1: return pick_nt<F16, 1, WT, PAIRWISE, KEEP, 1>(s, a, grid, st);
        case 1 * 8 + 2: return pick_nt<F16, 1, WT, PAIRWISE, KEEP, 2>(s, a, grid, st);
        case 1 * 8 + 4: return pick_nt<F16, 1, WT, PAIRWISE, KEEP, 4>(s, a, grid, st);
        default: return hipErrorInvalidValue;
    }
}

template <bool F16, int WT>
hipError_t pick_order_keep(const KvKernelSel& s, const KvLaunchArgs& a, unsigned grid, hipStream_t st) {
    if (s.pairwise) return s.keep_sum ? pick_shape<F16, WT, true, true>(s, a, grid, st) : pick_shape<F16, WT, true, false>(s, a, grid, st);
    return s.keep_sum ? pick_shape<F16, WT, false, true>(s, a, grid, st) : pick_shape<F16, WT, false, false>(s, a, grid, st);
}

}  // namespace

#define KV_CAT2(a, b, c, d) a##b##c##d
#define KV_CAT(a, b, c, d) KV_CAT2(a, b, c, d)

hipError_t KV_CAT(kv_launch_fused_f, KV_TU_F16, _w, KV_TU_W)(const KvKernelSel& sel, const KvLaunchArgs& args,
                                                             unsigned grid, hipStream_t stream) {
    return pick_order_keep<(KV_TU_F16 != 0), KV_TU_W>(sel, args, grid, stream);
}
