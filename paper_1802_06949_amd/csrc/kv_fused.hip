// Fused W-way gradient reduction + scale + momentum-SGD update for gfx950.
//
// This translation unit is compiled once per (gradient dtype, W) pair, selected
// by -DKV_TU_F16={0,1} and -DKV_TU_W={0,2,4,8,16,32} (0 = W known only at run
// time), and exports one launcher, kv_launch_fused_f<F16>_w<W>.
//
// The path is a pure streaming pass: per parameter element it reads W gradient
// values once, reads w and m, and writes w' and m'.  There is no reuse, so there
// is no LDS staging and no MFMA; what matters is that every lane issues
// independent vector loads (128 bits of fp32 or 64 bits of fp16 gradients per rank; all W
// ranks, and `U` vectors per rank, are in flight before the first add) and that a
// wavefront's 64 lanes cover contiguous memory per load instruction.
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

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

template <bool F16> struct Grad;
template <> struct Grad<false> {
    using elem = float;
    using vec = f32x4;
    static constexpr int VEC = 4;
    static __device__ __forceinline__ void widen(const vec& v, float (&o)[4]) {
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
    static __device__ __forceinline__ float widen1(elem e) { return e; }
};
// Half-precision gradients are read 8 bytes (4 values) per lane, not 16: a lane then owns 4
// consecutive elements, exactly one 16-byte vector of w and of m, so that every load and store of
// the fp32 state covers whole cache lines.  (With 8 halves per lane the state accesses of a
// wavefront touch every line half, twice; measured 9 % slower on ResNet-50 W=32.)
template <> struct Grad<true> {
    using elem = _Float16;
    using vec = f16x4;
    static constexpr int VEC = 4;
    static __device__ __forceinline__ void widen(const vec& v, float (&o)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = (float)v[i];      // exact: every binary16 value is a binary32 value
    }
    static __device__ __forceinline__ float widen1(elem e) { return (float)e; }
};

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
template <bool NT>
__device__ __forceinline__ f32x4 load_state(const float* p) {
    if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    else return *reinterpret_cast<const f32x4*>(p);
}
// Stores 16 bytes at element `k` of the uniform base pointer `base`.  Policy 8 uses a raw
// buffer store, whose cache-policy operand can carry the sc1 bit (write through L2 to memory
// at once instead of leaving a dirty line in L2); the buffer descriptor spans exactly the
// bytes handed in, so an out-of-range lane could not write.  0x00020000 is word 3 of a raw
// (untyped, 32-bit data format) buffer descriptor on gfx9-family targets.
template <int POL>
__device__ __forceinline__ void store_state(float* base, int k, unsigned span_bytes, const f32x4& v) {
    if constexpr (POL == 4) {
        __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(base + k));
    } else if constexpr (POL == 8 || POL == 12) {
        typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(base, 0, span_bytes, 0x00020000);
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), rsrc, k * 4, 0,
                                               POL == 12 ? /*sc1 + nt*/ 18 : /*sc1*/ 16);
    } else {
        *reinterpret_cast<f32x4*>(base + k) = v;
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

// Sum over ranks of the gradient vector (4 values) that starts `boff` bytes into every rank's copy of the key.
template <bool F16, int WT, bool PAIRWISE, bool NT>
__device__ __forceinline__ void reduce_vec(const uint64_t KV_CONST* gp, int W, int64_t boff,
                                           float (&s)[Grad<F16>::VEC]) {
    using G = Grad<F16>;
    using V = typename G::vec;
    constexpr int NV = G::VEC;
    typename FoldSel<NV, PAIRWISE>::type f;
    if constexpr (WT > 0) {
        constexpr int CH = WT > 16 ? 16 : WT;      // ranks whose loads are issued back to back
#pragma unroll
        for (int r0 = 0; r0 < WT; r0 += CH) {
            V g[CH];
#pragma unroll
            for (int j = 0; j < CH; ++j) g[j] = load_grad<NT>((const V KV_GLOBAL*)(gp[r0 + j] + (uint64_t)boff));
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                float t[NV];
                G::widen(g[j], t);
                f.push(t);
            }
        }
    } else {
        for (int r0 = 0; r0 < W; r0 += 4) {
            V g[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (r0 + j < W) g[j] = load_grad<NT>((const V KV_GLOBAL*)(gp[r0 + j] + (uint64_t)boff));
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (r0 + j < W) {
                    float t[NV];
                    G::widen(g[j], t);
                    f.push(t);
                }
            }
        }
    }
    f.finish(s);
}

// Same for the single element `e` of the key (ragged tails and gradient buffers
// that are not 16-byte aligned).
template <bool F16, int WT, bool PAIRWISE>
__device__ __forceinline__ float reduce_one(const uint64_t KV_CONST* gp, int W, int64_t e) {
    using G = Grad<F16>;
    using E = typename G::elem;
    typename FoldSel<1, PAIRWISE>::type f;
    const int n = WT > 0 ? WT : W;
    for (int r = 0; r < n; ++r) {
        float t[1] = {G::widen1(((const E KV_GLOBAL*)gp[r])[e])};
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
// the same pass.  row == nullptr or a null first pointer: the key has no replicas.
struct Bcast {
    const uint64_t KV_CONST* row;
    int n;
    int f16;
};

__device__ __forceinline__ void bcast4(const Bcast& b, int64_t e, const f32x4& wn) {
    if (b.n == 0) return;
    if (b.f16) {
        f16x4 h;
#pragma unroll
        for (int c = 0; c < 4; ++c) h[c] = (_Float16)wn[c];
        for (int r = 0; r < b.n; ++r) *(f16x4 KV_GLOBAL*)(b.row[r] + (uint64_t)e * 2u) = h;
    } else {
        for (int r = 0; r < b.n; ++r) *(f32x4 KV_GLOBAL*)(b.row[r] + (uint64_t)e * 4u) = wn;
    }
}

__device__ __forceinline__ void bcast1(const Bcast& b, int64_t e, float wn) {
    if (b.n == 0) return;
    if (b.f16) {
        for (int r = 0; r < b.n; ++r) ((_Float16 KV_GLOBAL*)b.row[r])[e] = (_Float16)wn;
    } else {
        for (int r = 0; r < b.n; ++r) ((float KV_GLOBAL*)b.row[r])[e] = wn;
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

// Updates the four elements k..k+3 of the tile whose arenas start at wp / mp / sp.
template <bool KEEP, int NTS>
__device__ __forceinline__ void update_store4(const float* s4, const f32x4& wv, const f32x4& mv, float* wp, float* mp,
                                              float* sp, int k, unsigned span_bytes, const Bcast& bc, int64_t e,
                                              const KvLaunchArgs& a) {
    f32x4 wn, mn, sv;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        float wo, mo;
        sgd_update(s4[c], wv[c], mv[c], a.rescale, a.lr, a.momentum, a.wd, wo, mo);
        wn[c] = wo; mn[c] = mo; sv[c] = s4[c];
    }
    if constexpr (KEEP) store_state<NTS>(sp, k, span_bytes, sv);
    store_state<NTS>(mp, k, span_bytes, mn);
    store_state<NTS>(wp, k, span_bytes, wn);
    bcast4(bc, e, wn);
}

template <bool F16, int WT, bool PAIRWISE, bool KEEP, int U, int NTM>
__global__ void __launch_bounds__(KV_THREADS) kv_fused(const KvLaunchArgs a) {
    using G = Grad<F16>;
    using E = typename G::elem;
    constexpr int NV = G::VEC;
    constexpr int Q = NV / 4;                // float4 pieces of w / m per gradient vector
    constexpr int TILE = KV_THREADS * NV * U;
    constexpr bool NT = (NTM & 1) != 0;      // gradient loads
    constexpr bool NTL = (NTM & 2) != 0;     // w, m loads
    constexpr int NTS = NTM & 12;            // store policy of w', m', s
    const int W = WT > 0 ? WT : a.W;
    const int tid = threadIdx.x;

    // a KvTile as four 64-bit words: {seg | count << 32, arena_off, seg_off, reserved}
    static_assert(sizeof(KvTile) == 32, "tile layout");
    const int64_t KV_CONST* tiles = (const int64_t KV_CONST*)a.tiles + a.tile_lo * 4;
    const uint64_t KV_CONST* table = (const uint64_t KV_CONST*)a.gptrs;

    const int64_t ntiles = a.tile_hi - a.tile_lo;
    // The hardware deals consecutive workgroup ids round-robin to the 8 XCDs.  xcd_remap = 1 sends
    // them to 8 contiguous tile ranges, one per XCD; xcd_remap = G > 1 gives every XCD blocks of G
    // consecutive tiles (rows of 8 G tiles, block x of a row to XCD x); 0 leaves the tiles dealt
    // one by one.
    const int64_t blk = a.xcd_remap == 1 ? (ntiles + 7) >> 3 : a.xcd_remap;
    const int64_t span = a.xcd_remap ? (ntiles + 8 * blk - 1) / (8 * blk) * (8 * blk) : ntiles;

    for (int64_t i = blockIdx.x; i < span; i += gridDim.x) {
        int64_t t = i;
        if (a.xcd_remap) {
            const int64_t row = i / (8 * blk), within = i - row * (8 * blk);
            t = row * (8 * blk) + (within & 7) * blk + (within >> 3);
            if (t >= ntiles) continue;
        }
        struct { int32_t seg, count; int64_t arena_off, seg_off; } td;
        {
            const int64_t KV_CONST* tw = tiles + t * 4;
            const int64_t w0 = tw[0];
            td.seg = (int32_t)(w0 & 0xFFFFFFFF);
            td.count = (int32_t)(w0 >> 32);
            td.arena_off = tw[1];
            td.seg_off = tw[2];
        }
        float* __restrict__ wp = a.w + td.arena_off;
        float* __restrict__ mp = a.m + td.arena_off;
        float* __restrict__ sp = KEEP ? a.s + td.arena_off : nullptr;
        const uint64_t KV_CONST* gp = table + (int64_t)td.seg * W;
        const bool full = td.count == TILE;
        const unsigned span_bytes = (unsigned)td.count * 4u;      // bytes of this tile in each arena

        // A full tile lies wholly inside the arena, so its w and m vectors can be requested
        // before the gradient pointers have arrived (they are dropped in the rare case that
        // the gradient buffers turn out not to be 16-byte aligned).
        f32x4 w4[U][Q], m4[U][Q];
        if (full) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int k = (tid + u * KV_THREADS) * NV;
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    w4[u][q] = load_state<NTL>(wp + k + 4 * q);
                    m4[u][q] = load_state<NTL>(mp + k + 4 * q);
                }
            }
        }

        // The vector path needs every gradient pointer aligned to one gradient vector (16 bytes of
        // fp32, 8 bytes of fp16) and every replica pointer to one replica vector (16 or 8 bytes).
        uint64_t bits = 0;
        for (int r = 0; r < W; ++r) bits |= gp[r];
        bool vec_ok = (bits & (uint64_t)(NV * sizeof(E) - 1)) == 0;

        Bcast bc{nullptr, 0, a.bcast_f16};
        if (a.bcast_n > 0) {
            const uint64_t KV_CONST* row = (const uint64_t KV_CONST*)a.bcast + (int64_t)td.seg * a.bcast_n;
            if (row[0] != 0) {
                bc.row = row;
                bc.n = a.bcast_n;
                uint64_t rbits = 0;
                for (int r = 0; r < a.bcast_n; ++r) rbits |= row[r];
                vec_ok = vec_ok && (rbits & (a.bcast_f16 ? 7u : 15u)) == 0;
            }
        }

        if (vec_ok && full) {
            // every gradient load of every unrolled vector is issued before the first store
            float s[U][NV];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t e = td.seg_off + (int64_t)(tid + u * KV_THREADS) * NV;
                reduce_vec<F16, WT, PAIRWISE, NT>(gp, W, e * (int64_t)sizeof(E), s[u]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int k = (tid + u * KV_THREADS) * NV;
#pragma unroll
                for (int q = 0; q < Q; ++q)
                    update_store4<KEEP, NTS>(&s[u][4 * q], w4[u][q], m4[u][q], wp, mp, sp, k + 4 * q, span_bytes, bc,
                                             td.seg_off + k + 4 * q, a);
            }
        } else if (vec_ok) {
            // ragged tile: whole vectors first, then at most NV-1 single elements
            const int nvec = td.count / NV;
            for (int v = tid; v < nvec; v += KV_THREADS) {
                const int k = v * NV;
                float s[NV];
                reduce_vec<F16, WT, PAIRWISE, NT>(gp, W, (td.seg_off + k) * (int64_t)sizeof(E), s);
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    const f32x4 wv = load_state<NTL>(wp + k + 4 * q);
                    const f32x4 mv = load_state<NTL>(mp + k + 4 * q);
                    update_store4<KEEP, NTS>(&s[4 * q], wv, mv, wp, mp, sp, k + 4 * q, span_bytes, bc,
                                             td.seg_off + k + 4 * q, a);
                }
            }
            const int rem = td.count - nvec * NV;
            if (tid < rem) {
                const int k = nvec * NV + tid;
                scalar_element<F16, WT, PAIRWISE, KEEP>(gp, W, td.seg_off + k, k, wp, mp, sp, bc, a);
            }
        } else {
            for (int k = tid; k < td.count; k += KV_THREADS)
                scalar_element<F16, WT, PAIRWISE, KEEP>(gp, W, td.seg_off + k, k, wp, mp, sp, bc, a);
        }
    }
}

template <bool F16, int WT, bool PAIRWISE, bool KEEP, int U, int NTM>
hipError_t launch_one(const KvLaunchArgs& a, unsigned grid, hipStream_t st) {
    hipLaunchKernelGGL((kv_fused<F16, WT, PAIRWISE, KEEP, U, NTM>), dim3(grid), dim3(KV_THREADS), 0, st, a);
    return hipGetLastError();
}

template <bool F16, int WT, bool PAIRWISE, bool KEEP, int U>
hipError_t pick_nt(const KvKernelSel& s, const KvLaunchArgs& a, unsigned grid, hipStream_t st) {
    switch (s.nontemporal) {
        case 0: return launch_one<F16, WT, PAIRWISE, KEEP, U, 0>(a, grid, st);
        case 1: return launch_one<F16, WT, PAIRWISE, KEEP, U, 1>(a, grid, st);
        case 5: return launch_one<F16, WT, PAIRWISE, KEEP, U, 5>(a, grid, st);
        case 9: return launch_one<F16, WT, PAIRWISE, KEEP, U, 9>(a, grid, st);
        case 13: return launch_one<F16, WT, PAIRWISE, KEEP, U, 13>(a, grid, st);
        default: return hipErrorInvalidValue;
    }
}

template <bool F16, int WT, bool PAIRWISE, bool KEEP>
hipError_t pick_u(const KvKernelSel& s, const KvLaunchArgs& a, unsigned grid, hipStream_t st) {
    switch (s.unroll) {
        case 1: return pick_nt<F16, WT, PAIRWISE, KEEP, 1>(s, a, grid, st);
        case 2: return pick_nt<F16, WT, PAIRWISE, KEEP, 2>(s, a, grid, st);
        case 4: return pick_nt<F16, WT, PAIRWISE, KEEP, 4>(s, a, grid, st);
        default: return hipErrorInvalidValue;
    }
}

template <bool F16, int WT>
hipError_t pick_order_keep(const KvKernelSel& s, const KvLaunchArgs& a, unsigned grid, hipStream_t st) {
    if (s.pairwise) return s.keep_sum ? pick_u<F16, WT, true, true>(s, a, grid, st) : pick_u<F16, WT, true, false>(s, a, grid, st);
    return s.keep_sum ? pick_u<F16, WT, false, true>(s, a, grid, st) : pick_u<F16, WT, false, false>(s, a, grid, st);
}

}  // namespace

#define KV_CAT2(a, b, c, d) a##b##c##d
#define KV_CAT(a, b, c, d) KV_CAT2(a, b, c, d)

hipError_t KV_CAT(kv_launch_fused_f, KV_TU_F16, _w, KV_TU_W)(const KvKernelSel& sel, const KvLaunchArgs& args,
                                                             unsigned grid, hipStream_t stream) {
    return pick_order_keep<(KV_TU_F16 != 0), KV_TU_W>(sel, args, grid, stream);
}
