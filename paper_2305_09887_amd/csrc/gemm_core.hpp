// The tile-product kernel template of libtma with its operand views, epilogues and launcher; included by the
// translation units that instantiate it (the GraphSAGE transforms, the dense / GCN transforms).
//
// One kernel template serves every product: operands are described by small "view" structs that present
// concatenations ([H | M], [W_self ; W_neigh]), the ReLU mask and transposes as plain A[m][k], B[k][n], and by
// an epilogue struct.  Arithmetic: fp32 storage multiplies with v_mfma_f32_32x32x2_f32 (fp32 in, fp32
// accumulate), bf16 storage with v_mfma_f32_32x32x16_bf16 (see TileMath).
//
// Tiling.  128 x BN block tile, 4 wavefronts, each owning a (BM/WM) x (BN/WN) patch of 32x32 MFMA tiles; k is
// consumed in slabs of BK through two LDS buffers (one barrier per slab) while the next slab's global loads are
// in flight in registers.  Every operand keeps in LDS the orientation it has in HBM, so all global->LDS
// traffic is 16-byte loads and 16-byte LDS writes:
//   k-contiguous operand : LDS [mn][BK+4]; a lane fetches the k-values of its row with one 16-byte read (4 fp32
//                          values for 4 MFMAs, 8 bf16 values for one);
//   mn-contiguous operand: LDS [BK][MN+4]; a lane reads one element per k-value.
// Within a group of k-values (8 for fp32, 16 for bf16) the lanes of the upper half take the upper half of the
// group, from both operands (any bijection of k is allowed as long as A and B agree).  Blocks are persistent and
// numbered so that the tiles sharing operand rows land on the same die (XCD) and hit its L2.
#pragma once
#include "kernels.hpp"

#include <type_traits>

namespace tma {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Which products keep two slabs in flight in registers (and then run two blocks per compute unit, 256 registers):
// the ones bound by streaming their operands -- bf16 storage, and the weight gradient whose k runs over the nodes.
// Measured at n = 125,237 / 2,000,000 rows: bf16 forward 97 -> 79 us / 1.34 -> 1.06 ms, bf16 narrow input gradient
// 66 -> 48 us, fp32 weight gradient 188 -> 180 us / 2.76 -> 2.53 ms; the fp32 forward and input-gradient products,
// whose matrix work per slab is four times longer, lose 5 % with it and keep one slab and three blocks; so does the
// bf16 input-gradient product of the aggregate-first form (169 -> 190 us), which already runs two blocks per unit.
template <typename CT, bool kColSum, bool kRowAux = false>
struct DeepPrefetch {
    static constexpr bool value = (sizeof(CT) == 2 && !kRowAux) || kColSum;
};

constexpr int kPad = 4;   // LDS row padding in words: keeps 16-byte alignment, spreads banks
constexpr int kXcds = 8;  // MI355X: 8 accelerator dies, workgroups are dealt round-robin to them

__device__ __forceinline__ float4 zero4() { return make_float4(0.0f, 0.0f, 0.0f, 0.0f); }

// f(integral_constant<int, 0>), ..., f(integral_constant<int, N - 1>): a loop whose index is a constant in the body
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(std::integral_constant<int, N - 1>{});
    }
}

// An optional member of an operand view: kPacksBf16 + packed(raw) say that the view's Raw already holds four bf16
// values the way a bf16 tile keeps them in LDS (bits unchanged), so a bf16 product stores them as they are instead
// of widening and rounding them again (the same bits either way).
template <class View, class = void>
struct PacksBf16 : std::false_type {};
template <class View>
struct PacksBf16<View, std::void_t<decltype(View::kPacksBf16)>> : std::integral_constant<bool, View::kPacksBf16> {};

// ---------------------------------------------------------------------------
// Storage types.  T = float (fp32 storage) or uint16_t (bf16 storage).  The
// views hand every operand over as fp32 quads (bf16 widened exactly); TileMath
// decides what sits in LDS and which MFMA multiplies it.  Results are rounded
// to bf16 (nearest even) on store.
// ---------------------------------------------------------------------------
template <typename T>
struct Pack4;
template <>
struct Pack4<float> {
    typedef float4 Packed;  // 16 bytes
    static __device__ __forceinline__ Packed load(const float *p) { return *reinterpret_cast<const float4 *>(p); }
    static __device__ __forceinline__ float4 widen(const Packed &v) { return v; }
};
template <>
struct Pack4<uint16_t> {
    typedef uint2 Packed;  // 8 bytes
    static __device__ __forceinline__ Packed load(const uint16_t *p) { return *reinterpret_cast<const uint2 *>(p); }
    static __device__ __forceinline__ float4 widen(const Packed &v)
    {
        return make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xFFFF0000u), __uint_as_float(v.y << 16),
                           __uint_as_float(v.y & 0xFFFF0000u));
    }
};
__device__ __forceinline__ float widen1(const float *p) { return *p; }
__device__ __forceinline__ float widen1(const uint16_t *p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void narrow1(float *p, float v) { *p = v; }
__device__ __forceinline__ void narrow1(uint16_t *p, float v) { *p = f32_to_bf16(v); }

// ---------------------------------------------------------------------------
// Operand views.  A view presents its operand as X[mn][k].  Per thread and
// load slot the kernel calls prepare(mn) once per tile (everything that does
// not depend on k: row pointers, which half of a concatenation, validity), then
// load(lane, k) once per k-slab, which returns four consecutive elements along
// the view's contiguous direction (k when kContigK, else mn) as a Raw value;
// resolve(raw) turns it into fp32 operand values, zero outside the operand.
// The split lets the kernel issue the loads of the next slab before the MFMAs of
// the current one and touch the loaded registers (widening, ReLU mask, ragged
// tails) only afterwards, so no wait on global memory sits in front of the
// matrix work.  V = the vector path is legal (bases aligned to four elements,
// leading dimensions and inner extents multiples of 4); its loads are
// branch-free: an out-of-range position is clamped to a valid address and the
// value is discarded by resolve() through the `ok` flag.  Without V the view
// loads element by element, guarded (the side-weight views have a third way: see RawU).
// ---------------------------------------------------------------------------
template <typename T, bool V>
struct RawV {
    typename Pack4<T>::Packed v;
    bool ok;
    __device__ __forceinline__ float4 get() const
    {
        const float4 f = Pack4<T>::widen(v);
        return make_float4(ok ? f.x : 0.0f, ok ? f.y : 0.0f, ok ? f.z : 0.0f, ok ? f.w : 0.0f);
    }
};
template <typename T>
struct RawV<T, false> {  // element-wise path: already fp32, already zero outside
    float4 v;
    bool ok;
    __device__ __forceinline__ float4 get() const { return v; }
};

// Weight matrices whose rows are not multiples of four (F_out = 47): four consecutive elements starting at
// element e of a dense fp32 array of `count` >= 4 elements, fetched with one 16-byte load from a base that is
// only 4-byte aligned (the load instruction needs no more), unconditionally.  A group that would run past the
// end of the array is fetched `shift` elements earlier and moved back in registers; `valid` leading elements are
// kept, the rest read as zero.
struct RawU {
    float4 v;
    int meta;  // valid (0..4) | shift (0..3) << 4
    __device__ __forceinline__ float4 get() const
    {
        const int valid = meta & 15;
        float4 t = v;
        if (meta & 16) t = make_float4(t.y, t.z, t.w, 0.0f);
        if (meta & 32) t = make_float4(t.z, t.w, 0.0f, 0.0f);
        return make_float4(valid > 0 ? t.x : 0.0f, valid > 1 ? t.y : 0.0f, valid > 2 ? t.z : 0.0f, valid > 3 ? t.w : 0.0f);
    }
};
__device__ __forceinline__ RawU load_unaligned4(const float *base, int e, int count, int valid)
{
    const int over = e + 4 - count;
    const int shift = over > 0 ? over : 0;
    RawU r;
    __builtin_memcpy(&r.v, base + (e - shift), 16);
    r.meta = (valid < 4 ? valid : 4) | (shift << 4);
    return r;
}
enum : int { kElementwise = 0, kAligned4 = 1, kUnaligned4 = 2 };   // how a weight view fetches its groups of four

template <typename T, bool V>
struct CatRows {  // A[m][k] = k < F ? H[m][k] : M[m][k-F]  for k < Kv, zero beyond    (contiguous along k)
    static constexpr bool kContigK = true;
    typedef RawV<T, V> Raw;
    struct Lane {
        const T *p0, *p1;  // row pointers such that element k is p0[k] (k < F) or p1[k] (k >= F)
        bool ok;
    };
    const T *H;
    int64_t ldh;
    const T *Mx;
    int64_t ldm;
    int F;
    int64_t rows;
    int Kv;  // extent of k: 2F for the concatenation, F when only the first part is used (Mx is then never read)
    static __device__ __forceinline__ float4 resolve(const Raw &r) { return r.get(); }
    static constexpr bool kPacksBf16 = V && sizeof(T) == 2;
    static __device__ __forceinline__ uint2 packed(const Raw &r)
    {
        if constexpr (kPacksBf16) return make_uint2(r.ok ? r.v.x : 0u, r.ok ? r.v.y : 0u);
        else return make_uint2(0u, 0u);
    }
    __device__ __forceinline__ Lane prepare(int64_t m) const
    {
        const int64_t mm = m < rows ? m : 0;
        return Lane{H + mm * ldh, Mx + mm * ldm - F, m < rows};
    }
    __device__ __forceinline__ float at(const Lane &l, int k) const
    {
        return k < Kv ? (k < F ? widen1(l.p0 + k) : widen1(l.p1 + k)) : 0.0f;
    }
    __device__ __forceinline__ Raw load(const Lane &l, int64_t k64) const
    {
        const int k = int(k64);
        Raw r;
        r.ok = l.ok && k < Kv;
        if constexpr (V) {
            const int kc = k < Kv ? k : 0;
            r.v = Pack4<T>::load((kc < F ? l.p0 : l.p1) + kc);
        } else {
            r.v = r.ok ? make_float4(at(l, k), at(l, k + 1), at(l, k + 2), at(l, k + 3)) : zero4();
        }
        return r;
    }
    __device__ __forceinline__ bool k_plain() const { return V; }
    __device__ __forceinline__ Raw load_plain(const Lane &l, int64_t k64) const
    {
        if constexpr (V) {
            const int k = int(k64);
            Raw r;
            r.ok = l.ok;
            r.v = Pack4<T>::load((k < F ? l.p0 : l.p1) + k);
            return r;
        } else {
            return load(l, k64);
        }
    }
};

template <typename T, bool V>
struct CatRowsT {  // A[m][k] = (m < F ? H[k][m] : M[k][m-F])          (contiguous along m); k = node
    static constexpr bool kContigK = false;
    typedef RawV<T, V> Raw;
    struct Lane {
        const T *p;  // column pointer: element of node k is p[k * ld]
        int64_t ld;
        int m;
        bool ok;
    };
    const T *H;
    int64_t ldh;
    const T *Mx;
    int64_t ldm;
    int F;
    int64_t rows;
    static __device__ __forceinline__ float4 resolve(const Raw &r) { return r.get(); }
    __device__ __forceinline__ Lane prepare(int64_t m64) const
    {
        const int m = int(m64);
        if (m < F) return Lane{H + m, ldh, m, true};
        return Lane{Mx + (m < 2 * F ? m - F : 0), ldm, m, m < 2 * F};
    }
    __device__ __forceinline__ float at(int64_t node, int m) const
    {
        if (m < F) return widen1(H + node * ldh + m);
        if (m < 2 * F) return widen1(Mx + node * ldm + (m - F));
        return 0.0f;
    }
    __device__ __forceinline__ Raw load(const Lane &l, int64_t node) const
    {
        Raw r;
        r.ok = l.ok && node < rows;
        if constexpr (V) {
            r.v = Pack4<T>::load(l.p + (node < rows ? node : 0) * l.ld);
        } else {
            r.v = r.ok ? make_float4(at(node, l.m), at(node, l.m + 1), at(node, l.m + 2), at(node, l.m + 3)) : zero4();
        }
        return r;
    }
    __device__ __forceinline__ bool k_plain() const { return V; }
    __device__ __forceinline__ Raw load_plain(const Lane &l, int64_t node) const
    {
        if constexpr (V) {
            Raw r;
            r.ok = l.ok;
            r.v = Pack4<T>::load(l.p + node * l.ld);
            return r;
        } else {
            return load(l, node);
        }
    }
};

template <bool V>
struct CatWeights {  // B[k][n] = k < F ? W_self[k][n] : W_neigh[k-F][n]  (contiguous along n); fp32 master weights
    static constexpr bool kContigK = false;
    typedef RawV<float, V> Raw;
    struct Lane {
        int n;
    };
    const float *Ws;
    const float *Wn;
    int F;
    int N;
    static __device__ __forceinline__ float4 resolve(const Raw &r) { return r.get(); }
    __device__ __forceinline__ Lane prepare(int64_t n) const { return Lane{int(n)}; }
    __device__ __forceinline__ Raw load(const Lane &l, int64_t k64) const
    {
        const int n = l.n, k = int(k64);
        Raw r;
        r.ok = k < 2 * F && n < N;
        const int kc = k < 2 * F ? k : 0;
        const float *row = kc < F ? Ws + int64_t(kc) * N : Wn + int64_t(kc - F) * N;
        if constexpr (V) {
            r.v = *reinterpret_cast<const float4 *>(row + (n < N ? n : 0));
        } else if (r.ok) {
            r.v.x = row[n];
            r.v.y = n + 1 < N ? row[n + 1] : 0.0f;
            r.v.z = n + 2 < N ? row[n + 2] : 0.0f;
            r.v.w = n + 3 < N ? row[n + 3] : 0.0f;
        } else {
            r.v = zero4();
        }
        return r;
    }
    __device__ __forceinline__ bool k_plain() const { return V; }
    __device__ __forceinline__ Raw load_plain(const Lane &l, int64_t k64) const
    {
        if constexpr (V) {
            const int k = int(k64);
            Raw r;
            r.ok = l.n < N;
            const float *row = k < F ? Ws + int64_t(k) * N : Wn + int64_t(k - F) * N;
            r.v = *reinterpret_cast<const float4 *>(row + (l.n < N ? l.n : 0));
            return r;
        } else {
            return load(l, k64);
        }
    }
};

template <bool V>
struct CatWeightsT {  // B[k][n] = n < F ? W_self[n][k] : W_neigh[n-F][k]  (contiguous along k); k = output feature
    static constexpr bool kContigK = true;
    typedef RawV<float, V> Raw;
    struct Lane {
        const float *row;
        bool ok;
    };
    const float *Ws;
    const float *Wn;
    int F;
    int Fo;
    static __device__ __forceinline__ float4 resolve(const Raw &r) { return r.get(); }
    __device__ __forceinline__ Lane prepare(int64_t n64) const
    {
        const int n = int(n64);
        if (n < F) return Lane{Ws + int64_t(n) * Fo, true};
        return Lane{Wn + int64_t(n < 2 * F ? n - F : 0) * Fo, n < 2 * F};
    }
    __device__ __forceinline__ Raw load(const Lane &l, int64_t k64) const
    {
        const int k = int(k64);
        Raw r;
        r.ok = l.ok && k < Fo;
        if constexpr (V) {
            r.v = *reinterpret_cast<const float4 *>(l.row + (k < Fo ? k : 0));
        } else if (r.ok) {
            r.v.x = l.row[k];
            r.v.y = k + 1 < Fo ? l.row[k + 1] : 0.0f;
            r.v.z = k + 2 < Fo ? l.row[k + 2] : 0.0f;
            r.v.w = k + 3 < Fo ? l.row[k + 3] : 0.0f;
        } else {
            r.v = zero4();
        }
        return r;
    }
    __device__ __forceinline__ bool k_plain() const { return V; }
    __device__ __forceinline__ Raw load_plain(const Lane &l, int64_t k64) const
    {
        if constexpr (V) {
            Raw r;
            r.ok = l.ok;
            r.v = *reinterpret_cast<const float4 *>(l.row + k64);
            return r;
        } else {
            return load(l, k64);
        }
    }
};

// dZ = dHnext (.) [Hnext > 0] (ReLU) or dHnext (identity); rows = nodes, [rows, Fo] with leading dimension ld.
// kAsA: used as A[m=node][k=o] (contiguous along k).  Otherwise as B[k=node][n=o] (contiguous along n).
// The vector path may read up to three padding elements past Fo inside a row (ld is a multiple of 4);
// resolve() discards them.
template <bool kAsA, typename T, bool V, bool kRelu>
struct MaskedGrad {
    static constexpr bool kContigK = kAsA;
    typedef typename std::conditional<V, typename Pack4<T>::Packed, float4>::type Quad;
    struct RawRelu {
        Quad g, h;
        int nv;  // leading elements that are inside the operand (<= 0: none)
    };
    struct RawPlain {
        Quad g;
        int nv;
    };
    typedef typename std::conditional<kRelu, RawRelu, RawPlain>::type Raw;
    struct Lane {
        int64_t off;  // kAsA: node * ld ; else: o
        bool ok;
    };
    const T *dHn;
    const T *Hn;  // forward output; read only with ReLU
    int Fo;
    int64_t ld;
    int64_t rows;
    static __device__ __forceinline__ float4 quad(const Quad &q)
    {
        if constexpr (V) return Pack4<T>::widen(q);
        else return q;
    }
    static __device__ __forceinline__ float4 resolve(const Raw &r)
    {
        const float4 g = quad(r.g);
        if constexpr (kRelu) {
            const float4 h = quad(r.h);
            return make_float4((r.nv > 0 && h.x > 0.0f) ? g.x : 0.0f, (r.nv > 1 && h.y > 0.0f) ? g.y : 0.0f,
                               (r.nv > 2 && h.z > 0.0f) ? g.z : 0.0f, (r.nv > 3 && h.w > 0.0f) ? g.w : 0.0f);
        } else {
            return make_float4(r.nv > 0 ? g.x : 0.0f, r.nv > 1 ? g.y : 0.0f, r.nv > 2 ? g.z : 0.0f,
                               r.nv > 3 ? g.w : 0.0f);
        }
    }
    __device__ __forceinline__ Lane prepare(int64_t mn) const
    {
        if (kAsA) return Lane{(mn < rows ? mn : 0) * ld, mn < rows};
        return Lane{mn < Fo ? mn : 0, mn < Fo};
    }
    __device__ __forceinline__ Raw load(const Lane &l, int64_t k) const
    {
        Raw r;
        const int o = int(kAsA ? k : l.off);
        const bool inside = kAsA ? (l.ok && o < Fo) : (l.ok && k < rows);
        r.nv = inside ? Fo - o : 0;
        if constexpr (V) {
            const int64_t e = kAsA ? l.off + (o < Fo ? o : 0) : (k < rows ? k : 0) * ld + o;
            r.g = Pack4<T>::load(dHn + e);
            if constexpr (kRelu) r.h = Pack4<T>::load(Hn + e);
        } else {
            r.g = zero4();
            if constexpr (kRelu) r.h = zero4();
            if (inside) {
                const int64_t e = kAsA ? l.off + o : k * ld + o;
                r.g.x = widen1(dHn + e);
                if (o + 1 < Fo) r.g.y = widen1(dHn + e + 1);
                if (o + 2 < Fo) r.g.z = widen1(dHn + e + 2);
                if (o + 3 < Fo) r.g.w = widen1(dHn + e + 3);
                if constexpr (kRelu) {
                    r.h.x = widen1(Hn + e);
                    if (o + 1 < Fo) r.h.y = widen1(Hn + e + 1);
                    if (o + 2 < Fo) r.h.z = widen1(Hn + e + 2);
                    if (o + 3 < Fo) r.h.w = widen1(Hn + e + 3);
                }
            }
        }
        return r;
    }
    __device__ __forceinline__ bool k_plain() const { return V; }
    __device__ __forceinline__ Raw load_plain(const Lane &l, int64_t k) const
    {
        if constexpr (V) {
            Raw r;
            int64_t e;
            if (kAsA) {   // k = output feature, whole groups of four inside [0, Fo)
                r.nv = l.ok ? 4 : 0;
                e = l.off + k;
            } else {      // k = node
                r.nv = l.ok ? Fo - int(l.off) : 0;
                e = k * ld + l.off;
            }
            r.g = Pack4<T>::load(dHn + e);
            if constexpr (kRelu) r.h = Pack4<T>::load(Hn + e);
            return r;
        } else {
            return load(l, k);
        }
    }
};

// ---------------------------------------------------------------------------
// Views for the transform-before-aggregate form of the layer (F_out much smaller
// than F_in):  Y = H [W_self | W_neigh],  H' = act(Y_self + Abar Y_neigh + b).
// The two halves of the concatenation are padded to Fp = F_out rounded up to the
// 16-byte element count, so that a group of four never straddles the halves;
// positions c >= F_out inside a half read as zero.
// ---------------------------------------------------------------------------
template <int kMode>
struct SideWeights {  // B[k][n] = n < Fp ? W_self[k][n] : W_neigh[k][n-Fp]   (contiguous along n)
    static constexpr bool kContigK = false;
    static constexpr bool V = kMode == kAligned4;
    typedef typename std::conditional<kMode == kUnaligned4, RawU, RawV<float, V>>::type Raw;
    struct Lane {
        const float *col;  // element of row k is col[k * Fo]  (kUnaligned4: the matrix, and c = first column)
        int nv;            // valid elements from this column on (<= 0: padding)
        int c;
    };
    const float *Ws;
    const float *Wn;
    int F;   // rows (= F_in)
    int Fo;  // valid columns per half
    int Fp;  // padded columns per half
    static __device__ __forceinline__ float4 resolve(const Raw &r) { return r.get(); }
    __device__ __forceinline__ Lane prepare(int64_t n64) const
    {
        const int n = int(n64);
        const bool second = n >= Fp;
        const int c = n - (second ? Fp : 0);
        const bool ok = n < 2 * Fp && c < Fo;
        if constexpr (kMode == kUnaligned4) return Lane{second ? Wn : Ws, ok ? Fo - c : 0, ok ? c : 0};
        else return Lane{(second ? Wn : Ws) + (ok ? c : 0), ok ? Fo - c : 0, 0};
    }
    __device__ __forceinline__ Raw load(const Lane &l, int64_t k64) const
    {
        const int k = int(k64);
        if constexpr (kMode == kUnaligned4) {
            return load_unaligned4(l.col, (k < F ? k : 0) * Fo + l.c, F * Fo, (l.nv > 0 && k < F) ? l.nv : 0);
        } else {
            Raw r;
            r.ok = l.nv > 0 && k < F;
            const float *p = l.col + int64_t(k < F ? k : 0) * Fo;
            if constexpr (V) {
                r.v = *reinterpret_cast<const float4 *>(p);
            } else if (r.ok) {
                r.v.x = p[0];
                r.v.y = l.nv > 1 ? p[1] : 0.0f;
                r.v.z = l.nv > 2 ? p[2] : 0.0f;
                r.v.w = l.nv > 3 ? p[3] : 0.0f;
            } else {
                r.v = zero4();
            }
            return r;
        }
    }
    __device__ __forceinline__ bool k_plain() const { return V; }
    __device__ __forceinline__ Raw load_plain(const Lane &l, int64_t k64) const
    {
        if constexpr (V) {
            Raw r;
            r.ok = l.nv > 0;
            r.v = *reinterpret_cast<const float4 *>(l.col + k64 * Fo);
            return r;
        } else {
            return load(l, k64);
        }
    }
};

template <int kMode>
struct SideWeightsT {  // B[k][n] = k < Fp ? W_self[n][k] : W_neigh[n][k-Fp]   (contiguous along k); n = input feature
    static constexpr bool kContigK = true;
    static constexpr bool V = kMode == kAligned4;
    typedef typename std::conditional<kMode == kUnaligned4, RawU, RawV<float, V>>::type Raw;
    struct Lane {
        const float *rs, *rn;  // rows such that element k is rs[k] (first half) or rn[k] (second half)
        int row;               // first element of the row inside its matrix
        bool ok;
    };
    const float *Ws;
    const float *Wn;
    int F;  // rows of W (= F_in) = extent of n
    int Fo;
    int Fp;
    static __device__ __forceinline__ float4 resolve(const Raw &r) { return r.get(); }
    __device__ __forceinline__ Lane prepare(int64_t n64) const
    {
        const int n = int(n64 < F ? n64 : 0);
        return Lane{Ws + int64_t(n) * Fo, Wn + int64_t(n) * Fo - Fp, n * Fo, n64 < F};
    }
    __device__ __forceinline__ Raw load(const Lane &l, int64_t k64) const
    {
        const int k = int(k64);
        const bool second = k >= Fp;
        const int c = k - (second ? Fp : 0);
        const bool ok = l.ok && k < 2 * Fp && c < Fo;
        if constexpr (kMode == kUnaligned4) {
            return load_unaligned4(second ? Wn : Ws, l.row + (ok ? c : 0), F * Fo, ok ? Fo - c : 0);
        } else {
            Raw r;
            r.ok = ok;
            const float *p = (second ? l.rn : l.rs) + (r.ok ? k : (second ? Fp : 0));
            if constexpr (V) {
                r.v = *reinterpret_cast<const float4 *>(p);
            } else if (r.ok) {
                r.v.x = p[0];
                r.v.y = c + 1 < Fo ? p[1] : 0.0f;
                r.v.z = c + 2 < Fo ? p[2] : 0.0f;
                r.v.w = c + 3 < Fo ? p[3] : 0.0f;
            } else {
                r.v = zero4();
            }
            return r;
        }
    }
    // without padding columns inside the halves every group of four along k is whole
    __device__ __forceinline__ bool k_plain() const { return V && Fo == Fp; }
    __device__ __forceinline__ Raw load_plain(const Lane &l, int64_t k64) const
    {
        if constexpr (V) {
            const int k = int(k64);
            Raw r;
            r.ok = l.ok;
            r.v = *reinterpret_cast<const float4 *>((k >= Fp ? l.rn : l.rs) + k);
            return r;
        } else {
            return load(l, k64);
        }
    }
};

// [dZ | dYn]: first half = dHnext (.) act'(Hnext) (leading dimension ld, Fo valid columns),
// second half = dYn (leading dimension ldy, Fp columns, padding already zero).
// kAsA: A[m=node][k] (contiguous along k); otherwise B[k=node][n] (contiguous along n).
template <bool kAsA, typename T, bool V, bool kRelu>
struct SideGrad {
    static constexpr bool kContigK = kAsA;
    typedef typename std::conditional<V, typename Pack4<T>::Packed, float4>::type Quad;
    struct Raw {
        Quad g, h;
        int nv;
        bool second;
    };
    struct Lane {
        int64_t a, b;  // kAsA: node*ld, node*ldy ; else: column inside its half, unused
        bool ok, second;
    };
    const T *dHn;
    const T *Hn;
    const T *dYn;
    int Fo, Fp;
    int64_t ld, ldy;
    int64_t rows;
    static __device__ __forceinline__ float4 quad(const Quad &q)
    {
        if constexpr (V) return Pack4<T>::widen(q);
        else return q;
    }
    static __device__ __forceinline__ float4 resolve(const Raw &r)
    {
        const float4 g = quad(r.g);
        bool o0 = r.nv > 0, o1 = r.nv > 1, o2 = r.nv > 2, o3 = r.nv > 3;
        if constexpr (kRelu) {
            const float4 h = quad(r.h);
            o0 = o0 && (r.second || h.x > 0.0f);
            o1 = o1 && (r.second || h.y > 0.0f);
            o2 = o2 && (r.second || h.z > 0.0f);
            o3 = o3 && (r.second || h.w > 0.0f);
        }
        return make_float4(o0 ? g.x : 0.0f, o1 ? g.y : 0.0f, o2 ? g.z : 0.0f, o3 ? g.w : 0.0f);
    }
    __device__ __forceinline__ Lane prepare(int64_t mn) const
    {
        if (kAsA) {
            const int64_t node = mn < rows ? mn : 0;
            return Lane{node * ld, node * ldy, mn < rows, false};
        }
        const bool second = mn >= Fp;
        const int64_t c = mn - (second ? Fp : 0);
        const bool ok = mn < 2 * Fp && (second || c < Fo);
        return Lane{ok ? c : 0, 0, ok, second};
    }
    __device__ __forceinline__ Raw load(const Lane &l, int64_t k) const
    {
        Raw r;
        bool second, inside;
        int c;
        int64_t eg, ey;
        if (kAsA) {
            second = k >= Fp;
            c = int(k - (second ? Fp : 0));
            inside = l.ok && k < 2 * Fp && (second || c < Fo);
            if (!inside) c = 0;
            eg = l.a + c;
            ey = l.b + c;
        } else {
            second = l.second;
            c = int(l.a);
            inside = l.ok && k < rows;
            const int64_t node = k < rows ? k : 0;
            eg = node * ld + c;
            ey = node * ldy + c;
        }
        r.second = second;
        r.nv = inside ? (second ? Fp : Fo) - c : 0;
        if constexpr (V) {
            r.g = Pack4<T>::load(second ? dYn + ey : dHn + eg);
            if constexpr (kRelu) r.h = Pack4<T>::load(Hn + eg);
            else r.h = r.g;
        } else {
            r.g = zero4();
            r.h = zero4();
            if (inside) {
                const T *pg = second ? dYn + ey : dHn + eg;
                const int lim = r.nv;
                r.g.x = widen1(pg);
                if (lim > 1) r.g.y = widen1(pg + 1);
                if (lim > 2) r.g.z = widen1(pg + 2);
                if (lim > 3) r.g.w = widen1(pg + 3);
                if (kRelu && !second) {
                    const T *ph = Hn + eg;
                    r.h.x = widen1(ph);
                    if (lim > 1) r.h.y = widen1(ph + 1);
                    if (lim > 2) r.h.z = widen1(ph + 2);
                    if (lim > 3) r.h.w = widen1(ph + 3);
                }
            }
        }
        return r;
    }
    __device__ __forceinline__ bool k_plain() const { return V && (!kAsA || Fo == Fp); }
    __device__ __forceinline__ Raw load_plain(const Lane &l, int64_t k) const
    {
        if constexpr (V) {
            Raw r;
            int64_t eg, ey;
            if (kAsA) {   // k = position in [dZ | dYn], no padding inside the halves
                r.second = k >= Fp;
                const int c = int(k - (r.second ? Fp : 0));
                r.nv = l.ok ? 4 : 0;
                eg = l.a + c;
                ey = l.b + c;
            } else {      // k = node
                r.second = l.second;
                const int c = int(l.a);
                r.nv = l.ok ? (r.second ? Fp : Fo) - c : 0;
                eg = k * ld + c;
                ey = k * ldy + c;
            }
            r.g = Pack4<T>::load(r.second ? dYn + ey : dHn + eg);
            if constexpr (kRelu) r.h = Pack4<T>::load(Hn + eg);
            else r.h = r.g;
            return r;
        } else {
            return load(l, k);
        }
    }
};

// ---------------------------------------------------------------------------
// Epilogues.  col_aux / row_aux are fetched once per tile column / row with a
// clamped (always valid) index; value() is pure arithmetic on registers.
// ---------------------------------------------------------------------------
// Two-byte results: an epilogue that can name the address of an element (at) and vouches that columns 2c and 2c + 1
// of a row are one aligned 4-byte word (pairs_ok) lets neighbouring lanes trade every other value, so that each
// lane stores two columns of one row in one instruction instead of one column of two rows in two.
template <class E, class = void>
struct StoresPairs : std::false_type {};
template <class E>
struct StoresPairs<E, std::void_t<decltype(&E::pairs_ok)>> : std::bool_constant<E::kPairs> {};

__device__ __forceinline__ bool word_aligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3) == 0; }

template <class E>
__device__ __forceinline__ bool pairs_ok_of(const E &e)
{
    if constexpr (StoresPairs<E>::value) return e.pairs_ok();
    else return false;
}
template <class E>
__device__ __forceinline__ void store_pair(const E &e, int64_t row, int col, uint32_t word)
{
    if constexpr (StoresPairs<E>::value) *reinterpret_cast<uint32_t *>(e.at(row, col)) = word;
}

template <typename T>
struct FwdEpilogue {  // H' = act(acc + b)
    static constexpr bool kColAux = true, kRowAux = false;
    T *out;
    int64_t ld;
    const float *bias;
    bool relu;
    __device__ __forceinline__ float col_aux(int col) const { return bias[col]; }
    __device__ __forceinline__ float row_aux(int64_t) const { return 0.0f; }
    __device__ __forceinline__ float value(float v, float caux, float, int) const
    {
        v += caux;
        if (relu) v = v > 0.0f ? v : 0.0f;
        return v;
    }
    __device__ __forceinline__ void store(int64_t row, int col, float v, int) const { narrow1(out + row * ld + col, v); }
    static constexpr bool kPairs = sizeof(T) == 2;
    __device__ __forceinline__ bool pairs_ok() const { return ld % 2 == 0 && word_aligned(out); }
    __device__ __forceinline__ T *at(int64_t row, int col) const { return out + row * ld + col; }
};

template <typename T>
struct BwdDataEpilogue {  // columns [0,F): dH_self (leading dimension ldh) ; [F,2F): inv_deg[row] * dM (dense)
    static constexpr bool kColAux = false, kRowAux = true;
    T *dH;
    int64_t ldh;
    T *dMs;
    const float *inv_deg;
    int F;
    __device__ __forceinline__ float col_aux(int) const { return 0.0f; }
    __device__ __forceinline__ float row_aux(int64_t row) const { return inv_deg[row]; }
    __device__ __forceinline__ float value(float v, float, float raux, int col) const { return col < F ? v : v * raux; }
    __device__ __forceinline__ void store(int64_t row, int col, float v, int) const
    {
        if (col < F) narrow1(dH + row * ldh + col, v);
        else narrow1(dMs + row * F + (col - F), v);
    }
    static constexpr bool kPairs = sizeof(T) == 2;
    __device__ __forceinline__ bool pairs_ok() const
    {
        return ldh % 2 == 0 && F % 2 == 0 && word_aligned(dH) && word_aligned(dMs);
    }
    __device__ __forceinline__ T *at(int64_t row, int col) const
    {
        return col < F ? dH + row * ldh + col : dMs + row * F + (col - F);
    }
};

template <typename T>
struct HalvesEpilogue {  // columns [0,Fp): Y_self ; [Fp,2Fp): Y_neigh ; both [rows, ldy]
    static constexpr bool kColAux = false, kRowAux = false;
    T *Ys;
    T *Yn;
    int64_t ldy;
    int Fp;
    __device__ __forceinline__ float col_aux(int) const { return 0.0f; }
    __device__ __forceinline__ float row_aux(int64_t) const { return 0.0f; }
    __device__ __forceinline__ float value(float v, float, float, int) const { return v; }
    __device__ __forceinline__ void store(int64_t row, int col, float v, int) const
    {
        if (col < Fp) narrow1(Ys + row * ldy + col, v);
        else narrow1(Yn + row * ldy + (col - Fp), v);
    }
    static constexpr bool kPairs = sizeof(T) == 2;
    __device__ __forceinline__ bool pairs_ok() const
    {
        return ldy % 2 == 0 && Fp % 2 == 0 && word_aligned(Ys) && word_aligned(Yn);
    }
    __device__ __forceinline__ T *at(int64_t row, int col) const
    {
        return col < Fp ? Ys + row * ldy + col : Yn + row * ldy + (col - Fp);
    }
};

template <typename T>
struct RowsEpilogue {  // plain [rows, ld] output
    static constexpr bool kColAux = false, kRowAux = false;
    T *out;
    int64_t ld;
    __device__ __forceinline__ float col_aux(int) const { return 0.0f; }
    __device__ __forceinline__ float row_aux(int64_t) const { return 0.0f; }
    __device__ __forceinline__ float value(float v, float, float, int) const { return v; }
    __device__ __forceinline__ void store(int64_t row, int col, float v, int) const { narrow1(out + row * ld + col, v); }
    static constexpr bool kPairs = sizeof(T) == 2;
    __device__ __forceinline__ bool pairs_ok() const { return ld % 2 == 0 && word_aligned(out); }
    __device__ __forceinline__ T *at(int64_t row, int col) const { return out + row * ld + col; }
};

struct SplitEpilogue {  // partial products, one slab per split
    static constexpr bool kColAux = false, kRowAux = false;
    float *partial;
    int64_t Mtot;
    int N;
    __device__ __forceinline__ float col_aux(int) const { return 0.0f; }
    __device__ __forceinline__ float row_aux(int64_t) const { return 0.0f; }
    __device__ __forceinline__ float value(float v, float, float, int) const { return v; }
    __device__ __forceinline__ void store(int64_t row, int col, float v, int split) const
    {
        partial[(int64_t(split) * Mtot + row) * N + col] = v;
    }
};

// ---------------------------------------------------------------------------
// Arithmetic of the tile product.  CT = float: operands sit in LDS as fp32 and a
// group of 8 k-values is four v_mfma_f32_32x32x2_f32.  CT = uint16_t: operands sit
// in LDS as bf16 (activations stored in bf16 pass through unchanged, fp32 weights
// are rounded to nearest even on their way in) and a group of 16 k-values is ONE
// v_mfma_f32_32x32x16_bf16, whose operand layout -- lane l holds row l%32 and the
// eight k-values 8*(l/32) .. +7 -- is the fp32 fragment's with twice the k-values, so
// tile layouts, loaders and epilogues are shared.  Accumulation is fp32 in both.
// ---------------------------------------------------------------------------
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// two fp32 values to a pair of bf16, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    floatx2 v;
    v[0] = lo;
    v[1] = hi;
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

template <typename CT>
struct TileMath;

template <>
struct TileMath<float> {
    static constexpr int kGroupK = 8;   // k-values per fragment: four MFMAs of two
    typedef float4 Frag;
    static __device__ __forceinline__ void put(float *dst, const float4 &v) { *reinterpret_cast<float4 *>(dst) = v; }
    static __device__ __forceinline__ Frag along(const float *p) { return *reinterpret_cast<const float4 *>(p); }
    static __device__ __forceinline__ Frag strided(const float *p, int ld)
    {
        return make_float4(p[0], p[ld], p[2 * ld], p[3 * ld]);
    }
    static __device__ __forceinline__ float value(const float *p) { return *p; }
    static __device__ __forceinline__ void mma(const Frag &a, const Frag &b, floatx16 &acc)
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
    }
};

template <>
struct TileMath<uint16_t> {
    // one v_mfma_f32_32x32x16_bf16 per group of 16 k-values: lane l holds row l%32 and the eight k-values
    // 8*(l/32) .. +7 (the instruction this chip adds; the 32x32x8 one runs at half its rate)
    static constexpr int kGroupK = 16;
    typedef bf16x8 Frag;
    static __device__ __forceinline__ void put(uint16_t *dst, const float4 &v)
    {
        *reinterpret_cast<uint2 *>(dst) = make_uint2(pack_bf16(v.x, v.y), pack_bf16(v.z, v.w));
    }
    static __device__ __forceinline__ void put_bits(uint16_t *dst, const uint2 &w) { *reinterpret_cast<uint2 *>(dst) = w; }
    static __device__ __forceinline__ Frag along(const uint16_t *p)   // (tile rows are 8-byte aligned, not 16)
    {
        const uint2 lo = *reinterpret_cast<const uint2 *>(p), hi = *reinterpret_cast<const uint2 *>(p + 4);
        return __builtin_bit_cast(Frag, make_uint4(lo.x, lo.y, hi.x, hi.y));
    }
    static __device__ __forceinline__ Frag strided(const uint16_t *p, int ld)
    {
        uint4 w;
        w.x = uint32_t(p[0]) | (uint32_t(p[ld]) << 16);
        w.y = uint32_t(p[2 * ld]) | (uint32_t(p[3 * ld]) << 16);
        w.z = uint32_t(p[4 * ld]) | (uint32_t(p[5 * ld]) << 16);
        w.w = uint32_t(p[6 * ld]) | (uint32_t(p[7 * ld]) << 16);
        return __builtin_bit_cast(Frag, w);
    }
    static __device__ __forceinline__ float value(const uint16_t *p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void mma(const Frag &a, const Frag &b, floatx16 &acc)
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
    }
};

// ---------------------------------------------------------------------------
// C[M,N] = A[M,K] B[K,N], k split into ranges of k_per_split, fp32 MFMA.
// Work item = (split, m-tile, n-tile), numbered split-major then m then n.
// Persistent blocks: the grid is 8 x (blocks per die); the block with id b sits
// on die b % 8 and walks the work items  die*per_die + b/8, + blocks_per_die, ...
// so that at any time the blocks of a die work on neighbouring items (the n-tiles
// of one row block, the output tiles of one node range) and share them in its L2.
// The first slab of a block's next tile is fetched before the results of the
// current one are written out, so that its latency passes behind the stores.
// A tile whose k range consists of whole slabs inside both operands runs a main
// loop with unguarded loads (addresses affine in k: one addition per load and
// slab instead of clamps and 64-bit multiplications); a tile that lies wholly
// inside the result is written out without per-element bounds tests, which also
// gives the compiler a fixed number of stores to count its waits against.
// ---------------------------------------------------------------------------
template <typename CT, int BM, int BN, int BK, int WM, int WN, bool kColSum, class AL, class BL, class Epi>
__global__ __launch_bounds__(WM *WN * 64, (BK * sizeof(CT) <= 64 && !Epi::kRowAux && !DeepPrefetch<CT, kColSum, Epi::kRowAux>::value ? 3 : 2)) void gemm_f32_kernel(AL a, BL b, Epi epi, int64_t M, int N, int64_t K,
                                                                 int64_t k_per_split, int n_tiles,
                                                                 int64_t tiles_per_split, int64_t total_work,
                                                                 float *__restrict__ colsum_partial)
{
    constexpr int NT = WM * WN * 64;
    constexpr bool kPrefetch2 = DeepPrefetch<CT, kColSum, Epi::kRowAux>::value && (BM / WM / 32) * (BN / WN / 32) <= 4;   // (8 accumulator tiles leave no registers for it)
    constexpr int kDepth = 2;   // slabs in flight in registers (3 and 4 measured: no faster for any product, the wide forward one slower)
    constexpr int TM = BM / WM / 32;
    constexpr int TN = BN / WN / 32;
    constexpr int A_Q = BM * BK / 4, B_Q = BN * BK / 4;   // 16-byte pieces of a slab
    constexpr int A_V = (A_Q + NT - 1) / NT;              // load slots per thread; when the pieces do not divide
    constexpr int B_V = (B_Q + NT - 1) / NT;              // evenly the last slots repeat the last piece (same value)
    using Math = TileMath<CT>;
    typedef typename Math::Frag Frag;
    constexpr int GK = Math::kGroupK;   // k-values per fragment: 8 = 4 fp32 MFMAs, 16 = one bf16 MFMA
    constexpr int KG = BK / GK;
    constexpr int A_LD = AL::kContigK ? BK + kPad : BM + kPad;
    constexpr int B_LD = BL::kContigK ? BK + kPad : BN + kPad;
    constexpr int A_WORDS = AL::kContigK ? BM * A_LD : BK * A_LD;
    constexpr int B_WORDS = BL::kContigK ? BN * B_LD : BK * B_LD;
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0 && BK % GK == 0, "tile shape");
    static_assert(!kColSum || !BL::kContigK, "column sums are taken from a [k][n] tile");
    static_assert(A_WORDS * sizeof(CT) >= BN * sizeof(float) && B_WORDS * sizeof(CT) >= BM * sizeof(float),
                  "epilogue staging fits");

    __shared__ __attribute__((aligned(16))) CT As[2][A_WORDS];
    __shared__ __attribute__((aligned(16))) CT Bs[2][B_WORDS];
    float *const a_aux = reinterpret_cast<float *>(&As[0][0]);   // per-column / per-row epilogue inputs
    float *const b_aux = reinterpret_cast<float *>(&Bs[0][0]);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int l31 = lane & 31;
    const int hi = lane >> 5;
    const int wave = tid >> 6;
    const int wm0 = (wave / WN) * (BM / WM);
    const int wn0 = (wave % WN) * (BN / WN);

    // loop-invariant positions of this thread's load slots inside a tile, and their LDS word offsets
    int a_mn[A_V], a_k[A_V], a_lds[A_V], b_mn[B_V], b_k[B_V], b_lds[B_V];
#pragma unroll
    for (int i = 0; i < A_V; ++i) {
        const int idx = (tid + i * NT) < A_Q ? (tid + i * NT) : A_Q - 1;
        a_mn[i] = AL::kContigK ? idx / (BK / 4) : (idx % (BM / 4)) * 4;
        a_k[i] = AL::kContigK ? (idx % (BK / 4)) * 4 : idx / (BM / 4);
        a_lds[i] = AL::kContigK ? a_mn[i] * A_LD + a_k[i] : a_k[i] * A_LD + a_mn[i];
    }
#pragma unroll
    for (int i = 0; i < B_V; ++i) {
        const int idx = (tid + i * NT) < B_Q ? (tid + i * NT) : B_Q - 1;
        b_mn[i] = BL::kContigK ? idx / (BK / 4) : (idx % (BN / 4)) * 4;
        b_k[i] = BL::kContigK ? (idx % (BK / 4)) * 4 : idx / (BN / 4);
        b_lds[i] = BL::kContigK ? b_mn[i] * B_LD + b_k[i] : b_k[i] * B_LD + b_mn[i];
    }

    const int64_t blocks_per_die = gridDim.x / kXcds;
    const int64_t per_die = (total_work + kXcds - 1) / kXcds;
    const int64_t die = blockIdx.x % kXcds;
    int64_t die_end = (die + 1) * per_die;
    if (die_end > total_work) die_end = total_work;

    struct Tile {
        int64_t m0;
        int n0, split;
        int64_t k_begin, k_end;
    };
    auto tile_of = [&](int64_t work) {
        Tile t;
        t.split = int(work / tiles_per_split);
        const int64_t tile = work % tiles_per_split;
        t.m0 = (tile / n_tiles) * BM;
        t.n0 = int(tile % n_tiles) * BN;
        t.k_begin = int64_t(t.split) * k_per_split;
        t.k_end = t.k_begin + k_per_split;
        if (t.k_end > K) t.k_end = K;
        return t;
    };

    typename AL::Lane alane[A_V];
    typename BL::Lane blane[B_V];
    // first slab of the tile that comes next; the slabs inside a tile's main loop have registers of their own
    typename AL::Raw afirst[A_V];
    typename BL::Raw bfirst[B_V];
    auto prepare = [&](const Tile &t) {
#pragma unroll
        for (int i = 0; i < A_V; ++i) alane[i] = a.prepare(t.m0 + a_mn[i]);
#pragma unroll
        for (int i = 0; i < B_V; ++i) blane[i] = b.prepare(t.n0 + b_mn[i]);
    };
    // guarded: any position, clamped and flagged; plain: the caller knows the whole slab lies inside the
    // operands' k range, so the addresses are affine in k and cost one addition per slab
    auto fetch = [&](int64_t kt, typename AL::Raw(&ar)[A_V], typename BL::Raw(&br)[B_V]) {
#pragma unroll
        for (int i = 0; i < A_V; ++i) ar[i] = a.load(alane[i], kt + a_k[i]);
#pragma unroll
        for (int i = 0; i < B_V; ++i) br[i] = b.load(blane[i], kt + b_k[i]);
    };
    auto fetch_plain = [&](int64_t kt, typename AL::Raw(&ar)[A_V], typename BL::Raw(&br)[B_V]) {
#pragma unroll
        for (int i = 0; i < A_V; ++i) ar[i] = a.load_plain(alane[i], kt + a_k[i]);
#pragma unroll
        for (int i = 0; i < B_V; ++i) br[i] = b.load_plain(blane[i], kt + b_k[i]);
    };
    auto stage = [&](int buf, const typename AL::Raw(&ar)[A_V], const typename BL::Raw(&br)[B_V]) {
#pragma unroll
        for (int i = 0; i < A_V; ++i) {
            if constexpr (sizeof(CT) == 2 && PacksBf16<AL>::value) Math::put_bits(&As[buf][a_lds[i]], AL::packed(ar[i]));
            else Math::put(&As[buf][a_lds[i]], AL::resolve(ar[i]));
        }
#pragma unroll
        for (int i = 0; i < B_V; ++i) {
            if constexpr (sizeof(CT) == 2 && PacksBf16<BL>::value) Math::put_bits(&Bs[buf][b_lds[i]], BL::packed(br[i]));
            else Math::put(&Bs[buf][b_lds[i]], BL::resolve(br[i]));
        }
    };
    // This lane's k-values of group g (the upper half of the wavefront holds the upper half of the group) of its
    // row/column.
    auto frag_a = [&](int buf, int g, int i) -> Frag {
        const int mn = wm0 + i * 32 + l31;
        const int k = g * GK + (GK / 2) * hi;
        if (AL::kContigK) return Math::along(&As[buf][mn * A_LD + k]);
        return Math::strided(&As[buf][k * A_LD + mn], A_LD);
    };
    auto frag_b = [&](int buf, int g, int j) -> Frag {
        const int mn = wn0 + j * 32 + l31;
        const int k = g * GK + (GK / 2) * hi;
        if (BL::kContigK) return Math::along(&Bs[buf][mn * B_LD + k]);
        return Math::strided(&Bs[buf][k * B_LD + mn], B_LD);
    };

    int64_t work = die * per_die + blockIdx.x / kXcds;
    if (work >= die_end) return;
    const bool views_plain = a.k_plain() && b.k_plain();
    Tile t = tile_of(work);
    prepare(t);
    fetch(t.k_begin, afirst, bfirst);
    while (true) {
        floatx16 acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
        float colsum = 0.0f;

        __syncthreads();  // the previous tile's epilogue has finished reading LDS
        stage(0, afirst, bfirst);
        __syncthreads();

        // one slab from LDS buffer `buf`: fragment reads one group ahead of the MFMAs that use them
        auto multiply = [&](int buf) {
            Frag fa[2][TM], fb[2][TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[0][i] = frag_a(buf, 0, i);
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[0][j] = frag_b(buf, 0, j);
#pragma unroll
            for (int g = 0; g < KG; ++g) {
                const int cur = g & 1, nxt = cur ^ 1;
                if (g + 1 < KG) {  // next group's fragments are in flight while this group's MFMAs run
#pragma unroll
                    for (int i = 0; i < TM; ++i) fa[nxt][i] = frag_a(buf, g + 1, i);
#pragma unroll
                    for (int j = 0; j < TN; ++j) fb[nxt][j] = frag_b(buf, g + 1, j);
                }
                if constexpr (sizeof(CT) == 4) {   // fp32: the four k-pairs in turn, round-robin over the output tiles
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int i = 0; i < TM; ++i)
#pragma unroll
                            for (int j = 0; j < TN; ++j) {
                                const float av = q == 0 ? fa[cur][i].x : q == 1 ? fa[cur][i].y : q == 2 ? fa[cur][i].z : fa[cur][i].w;
                                const float bv = q == 0 ? fb[cur][j].x : q == 1 ? fb[cur][j].y : q == 2 ? fb[cur][j].z : fb[cur][j].w;
                                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[i][j], 0, 0, 0);
                            }
                } else {
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j) Math::mma(fa[cur][i], fb[cur][j], acc[i][j]);
                }
            }
            if (kColSum && t.m0 == 0 && tid < BN) {
#pragma unroll
                for (int k = 0; k < BK; ++k) colsum += Math::value(&Bs[buf][k * B_LD + tid]);
            }
        };
        auto main_loop = [&](auto plain_tag) {
            constexpr bool kPlain = decltype(plain_tag)::value;
            if constexpr (kPlain && kPrefetch2) {
                // Two slabs in flight in registers beside the two in LDS: a slab's loads are issued two iterations
                // before it is staged.  One iteration's matrix work is far shorter than a memory round trip under
                // load, so with a single slab in flight every iteration ends up waiting for one.
                // (kDepth register sets: slab s >= 1 waits in set (s - 1) % kDepth)
                typename AL::Raw areg[kDepth][A_V];
                typename BL::Raw breg[kDepth][B_V];
                const int64_t n_slabs = (t.k_end - t.k_begin) / BK;
                static_for<kDepth>([&](auto d_tag) {
                    constexpr int D = decltype(d_tag)::value;
                    if (n_slabs > D + 1) fetch_plain(t.k_begin + (D + 1) * BK, areg[D], breg[D]);
                });
                int buf = 0;
                for (int64_t sl0 = 0; sl0 < n_slabs; sl0 += kDepth) {
                    static_for<kDepth>([&](auto r_tag) {
                        constexpr int R = decltype(r_tag)::value;
                        const int64_t sl = sl0 + R;
                        if (sl < n_slabs) {      // the same for every thread
                            multiply(buf);
                            if (sl + 1 < n_slabs) stage(buf ^ 1, areg[R], breg[R]);
                            if (sl + 1 + kDepth < n_slabs) fetch_plain(t.k_begin + (sl + 1 + kDepth) * BK, areg[R], breg[R]);
                            __syncthreads();
                            buf ^= 1;
                        }
                    });
                }
            } else {
                typename AL::Raw areg[A_V];
                typename BL::Raw breg[B_V];
                int buf = 0;
                for (int64_t kt = t.k_begin; kt < t.k_end; kt += BK) {
                    const bool more = kt + BK < t.k_end;
                    if (more) {  // in flight while this slab is multiplied
                        if constexpr (kPlain) fetch_plain(kt + BK, areg, breg);
                        else fetch(kt + BK, areg, breg);
                    }
                    multiply(buf);
                    if (more) stage(buf ^ 1, areg, breg);  // the other buffer was last read before the previous barrier
                    __syncthreads();
                    buf ^= 1;
                }
            }
        };
        if (views_plain && (t.k_end - t.k_begin) % BK == 0) main_loop(std::true_type{});
        else main_loop(std::false_type{});

        // Per-column / per-row epilogue inputs (bias, 1/deg) go through LDS: they are loaded from
        // global memory once, here, before any store is in flight.  Fetched into registers directly they
        // would make the compiler guard every store below with a wait on the memory counter, which
        // also waits for the earlier stores and serialises the whole write-out.
        if (Epi::kColAux && tid < BN) a_aux[tid] = epi.col_aux(t.n0 + tid < N ? t.n0 + tid : N - 1);
        if (Epi::kRowAux && tid < BM) b_aux[tid] = epi.row_aux(t.m0 + tid < M ? t.m0 + tid : M - 1);
        if (Epi::kColAux || Epi::kRowAux) __syncthreads();

        // The first slab of this block's next tile is fetched now, so that its latency passes while the
        // results below are written out.
        const Tile done = t;
        const float done_colsum = colsum;
        const int64_t next = work + blocks_per_die;
        const bool has_next = next < die_end;
        if (has_next) {
            t = tile_of(next);
            prepare(t);
            fetch(t.k_begin, afirst, bfirst);
        }

        // MFMA 32x32 result layout: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32.
        float caux[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) caux[j] = Epi::kColAux ? a_aux[wn0 + j * 32 + l31] : 0.0f;
        auto write_out = [&](auto inside_tag) {
            constexpr bool kInside = decltype(inside_tag)::value;   // the whole tile lies inside the result
            bool pairs = false;
            if constexpr (kInside && StoresPairs<Epi>::value) pairs = pairs_ok_of(epi);   // the same for every lane
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                float raux[16];
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    raux[r] = Epi::kRowAux ? b_aux[wm0 + i * 32 + 8 * (r / 4) + 4 * hi + (r % 4)] : 0.0f;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = done.n0 + wn0 + j * 32 + l31;
                    if constexpr (kInside && StoresPairs<Epi>::value) {
                        if (pairs) {
                            // registers r and r + 1 are rows R and R + 1 of this lane's column: an odd lane gives its
                            // row-R value to the even lane on its left and gets that lane's row-R+1 value, so the
                            // even lane holds (col, col + 1) of row R and the odd one (col - 1, col) of row R + 1
                            const int odd = l31 & 1;
#pragma unroll
                            for (int r = 0; r < 16; r += 2) {
                                const int64_t row = done.m0 + wm0 + i * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
                                const float v0 = epi.value(acc[i][j][r], caux[j], raux[r], col);
                                const float v1 = epi.value(acc[i][j][r + 1], caux[j], raux[r + 1], col);
                                const float got = __shfl_xor(odd ? v0 : v1, 1, kWave);
                                const uint32_t word = odd ? pack_bf16(got, v1) : pack_bf16(v0, got);
                                store_pair(epi, row + odd, col - odd, word);
                            }
                            continue;
                        }
                    }
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int64_t row = done.m0 + wm0 + i * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
                        const float val = epi.value(acc[i][j][r], caux[j], raux[r], col);
                        if (kInside || (row < M && col < N)) epi.store(row, col, val, done.split);
                    }
                }
            }
        };
        if (done.m0 + BM <= M && done.n0 + BN <= N) write_out(std::true_type{});
        else write_out(std::false_type{});
        if (kColSum && done.m0 == 0 && tid < BN && done.n0 + tid < N)
            colsum_partial[int64_t(done.split) * N + done.n0 + tid] = done_colsum;
        if (!has_next) break;
        work = next;
    }
}

template <typename T>
static bool vec4_ok(const T *p, int64_t ld) { return aligned(p, 4 * sizeof(T)) && ld % 4 == 0; }

template <int BM, int BN, int BK, int WM, int WN, bool kColSum, typename CT = float, class AL, class BL, class Epi>
static void launch_gemm(const char *name, const AL &a, const BL &b, const Epi &e, int64_t M, int N, int64_t K,
                        int64_t k_per_split, int n_splits, float *colsum_partial, hipStream_t s)
{
    if (M <= 0 || N <= 0 || K <= 0) return;   // an empty product: callers zero-fill what they need
    const int n_tiles = int(ceil_div(N, BN));
    const int64_t tiles = ceil_div(M, BM) * n_tiles;
    const int64_t total = tiles * n_splits;
    // resident blocks per compute unit follow from the kernel's LDS footprint (160 KB per unit) and its
    // register budget (launch bounds); 256 units in 8 dies
    constexpr int kLdsBytes = 2 * int(sizeof(CT)) * ((AL::kContigK ? BM * (BK + kPad) : BK * (BM + kPad)) + (BL::kContigK ? BN * (BK + kPad) : BK * (BN + kPad)));
    // the launch bound's second number is waves per SIMD: 3 or 2, i.e. that many blocks of four wavefronts per compute
    // unit, half as many (at least one) of eight
    constexpr int kWavesPerSimd = (BK * sizeof(CT) <= 64 && !Epi::kRowAux && kLdsBytes <= 53 * 1024 && !DeepPrefetch<CT, kColSum, Epi::kRowAux>::value) ? 3 : 2;
    constexpr int kByWaves = kWavesPerSimd * 4 / (WM * WN) > 0 ? kWavesPerSimd * 4 / (WM * WN) : 1;
    constexpr int kByLds = 160 * 1024 / kLdsBytes > 0 ? 160 * 1024 / kLdsBytes : 1;
    constexpr int kPerCu = kByWaves < kByLds ? kByWaves : kByLds;
    int64_t blocks_per_die = ceil_div(total, kXcds);
    if (blocks_per_die > 32 * kPerCu) blocks_per_die = 32 * kPerCu;
    TMA_TIMED(name, s);
    hipLaunchKernelGGL((gemm_f32_kernel<CT, BM, BN, BK, WM, WN, kColSum, AL, BL, Epi>), dim3(unsigned(blocks_per_die * kXcds)),
                       dim3(WM * WN * 64), 0, s, a, b, e, M, N, K, k_per_split, n_tiles, tiles, total, colsum_partial);
}

// Kernel names for the timing hook: <what>_<tile>[_bf16][_generic]; "generic" = a streaming operand is
// on the element-wise path (the name does not say how the weights are read: aligned groups, unaligned groups
// or element by element, which costs a transform-first product about a tenth of its time).
template <typename T>
static const char *kname(const char *f32_vec, const char *f32_gen, const char *bf16_vec, const char *bf16_gen, bool vec)
{
    if (sizeof(T) == 4) return vec ? f32_vec : f32_gen;
    return vec ? bf16_vec : bf16_gen;
}

// A product with few 128x128 output tiles (a sampled block, a small part) would leave compute units without a
// workgroup or with a single one: below this many tiles (256 compute units) the narrower tile is taken, for twice
// as many workgroups.
#ifndef TMA_GEMM_FEW_TILES
#define TMA_GEMM_FEW_TILES 384
#endif
constexpr int64_t kFewTiles = TMA_GEMM_FEW_TILES;
static inline bool few_tiles(int64_t M, int64_t N, int n_splits = 1)
{
    return ceil_div(M, int64_t(128)) * ceil_div(N, int64_t(128)) * n_splits < kFewTiles;
}

template <typename CT, int BK, bool kColSum, class AL, class BL, class Epi>
static void launch_by_width(const char *name, const AL &a, const BL &b, const Epi &e, int64_t M, int N, int64_t K,
                            int64_t kps, int n_splits, float *colsum, hipStream_t s)
{
    if (N <= 64 || few_tiles(M, N, n_splits)) launch_gemm<128, 64, BK, 4, 1, kColSum, CT>(name, a, b, e, M, N, K, kps, n_splits, colsum, s);
    else if (N <= 96) launch_gemm<128, 96, BK, 4, 1, kColSum, CT>(name, a, b, e, M, N, K, kps, n_splits, colsum, s);
    else launch_gemm<128, 128, BK, 2, 2, kColSum, CT>(name, a, b, e, M, N, K, kps, n_splits, colsum, s);
}


struct WeightSplit {
    int n_splits;
    int64_t k_per_split;
    size_t partial_bytes, colsum_bytes;
};

}  // namespace tma
