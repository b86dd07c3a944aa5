// Dense per-layer transform of the mean-aggregation GraphSAGE layer and its
// gradients, on the matrix cores (the only MFMA-bound part of the path):
//   forward   Z = [H | M] [W_self ; W_neigh] + b,  H' = act(Z)
//   backward  [dH_self | D^-1 dM] = dZ [W_self^T | W_neigh^T]
//             [dW_self ; dW_neigh] = [H | M]^T dZ,   db = 1^T dZ
// with dZ = dH' (.) act'(Z) formed while loading (chain rule as in the proof of
// the paper's Thm. 1).
//
// fp32 storage uses v_mfma_f32_32x32x2_f32 (fp32 in, fp32 accumulate), so the
// 1e-4 parity bound holds without any reduced-precision pass.  One kernel
// template serves the three products: operands are described by small loader
// structs that present the concatenations [H | M] / [W_self ; W_neigh], the
// ReLU mask and the transposes as plain A[m][k], B[k][n] views, and by an
// epilogue struct.  Tiles are staged through LDS in k-major order so that the
// 32 lanes of an MFMA operand read 32 consecutive words.
#include "kernels.hpp"

namespace tma {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kPad = 4;  // LDS row padding (words); keeps rows 16-byte aligned

// ---------------------------------------------------------------------------
// Operand views.  load4(mn, k) returns four consecutive elements along the
// view's contiguous direction (k when kContigK, else m/n), zero outside.
// ---------------------------------------------------------------------------
struct CatRows {  // A[m][k] = k < F ? H[m][k] : M[m][k-F]          (contiguous along k)
    static constexpr bool kContigK = true;
    const float *H;
    int64_t ldh;
    const float *Mx;
    int F;
    int64_t rows;
    bool vec;
    __device__ __forceinline__ float at(int64_t m, int k) const
    {
        if (k < F) return H[m * ldh + k];
        if (k < 2 * F) return Mx[m * int64_t(F) + (k - F)];
        return 0.0f;
    }
    __device__ __forceinline__ float4 load4(int64_t m, int64_t k64) const
    {
        const int k = int(k64);
        if (m >= rows) return make_float4(0, 0, 0, 0);
        if (vec) {
            if (k < F) return *reinterpret_cast<const float4 *>(H + m * ldh + k);
            if (k < 2 * F) return *reinterpret_cast<const float4 *>(Mx + m * int64_t(F) + (k - F));
            return make_float4(0, 0, 0, 0);
        }
        return make_float4(at(m, k), at(m, k + 1), at(m, k + 2), at(m, k + 3));
    }
};

struct CatRowsT {  // A[m][k] = (m < F ? H[k][m] : M[k][m-F])          (contiguous along m); k = node
    static constexpr bool kContigK = false;
    const float *H;
    int64_t ldh;
    const float *Mx;
    int F;
    int64_t rows;
    bool vec;
    __device__ __forceinline__ float at(int64_t node, int m) const
    {
        if (m < F) return H[node * ldh + m];
        if (m < 2 * F) return Mx[node * int64_t(F) + (m - F)];
        return 0.0f;
    }
    __device__ __forceinline__ float4 load4(int64_t m64, int64_t node) const
    {
        const int m = int(m64);
        if (node >= rows) return make_float4(0, 0, 0, 0);
        if (vec) {
            if (m < F) return *reinterpret_cast<const float4 *>(H + node * ldh + m);
            if (m < 2 * F) return *reinterpret_cast<const float4 *>(Mx + node * int64_t(F) + (m - F));
            return make_float4(0, 0, 0, 0);
        }
        return make_float4(at(node, m), at(node, m + 1), at(node, m + 2), at(node, m + 3));
    }
};

struct CatWeights {  // B[k][n] = k < F ? W_self[k][n] : W_neigh[k-F][n]  (contiguous along n)
    static constexpr bool kContigK = false;
    const float *Ws;
    const float *Wn;
    int F;
    int N;
    bool vec;
    __device__ __forceinline__ float4 load4(int64_t n64, int64_t k64) const
    {
        const int n = int(n64), k = int(k64);
        if (k >= 2 * F) return make_float4(0, 0, 0, 0);
        const float *row = k < F ? Ws + int64_t(k) * N : Wn + int64_t(k - F) * N;
        if (vec && n + 3 < N) return *reinterpret_cast<const float4 *>(row + n);
        float4 r;
        r.x = n + 0 < N ? row[n + 0] : 0.0f;
        r.y = n + 1 < N ? row[n + 1] : 0.0f;
        r.z = n + 2 < N ? row[n + 2] : 0.0f;
        r.w = n + 3 < N ? row[n + 3] : 0.0f;
        return r;
    }
};

struct CatWeightsT {  // B[k][n] = n < F ? W_self[n][k] : W_neigh[n-F][k]  (contiguous along k); k = output feature
    static constexpr bool kContigK = true;
    const float *Ws;
    const float *Wn;
    int F;
    int Fo;
    bool vec;
    __device__ __forceinline__ float4 load4(int64_t n64, int64_t k64) const
    {
        const int n = int(n64), k = int(k64);
        if (n >= 2 * F) return make_float4(0, 0, 0, 0);
        const float *row = n < F ? Ws + int64_t(n) * Fo : Wn + int64_t(n - F) * Fo;
        if (vec && k + 3 < Fo) return *reinterpret_cast<const float4 *>(row + k);
        float4 r;
        r.x = k + 0 < Fo ? row[k + 0] : 0.0f;
        r.y = k + 1 < Fo ? row[k + 1] : 0.0f;
        r.z = k + 2 < Fo ? row[k + 2] : 0.0f;
        r.w = k + 3 < Fo ? row[k + 3] : 0.0f;
        return r;
    }
};

// dZ = dHnext (.) [Hnext > 0] (ReLU) or dHnext (identity); rows = nodes, dense [rows, Fo].
// kAsA: used as A[m=node][k=o] (contiguous along k).  Otherwise as B[k=node][n=o] (contiguous along n).
template <bool kAsA>
struct MaskedGrad {
    static constexpr bool kContigK = kAsA;
    const float *dHn;
    const float *Hn;  // forward output; read only when relu
    int Fo;
    int64_t rows;
    bool relu;
    bool vec;
    __device__ __forceinline__ float at(int64_t node, int o) const
    {
        if (o >= Fo) return 0.0f;
        float g = dHn[node * Fo + o];
        if (relu && !(Hn[node * Fo + o] > 0.0f)) g = 0.0f;
        return g;
    }
    __device__ __forceinline__ float4 load4(int64_t a, int64_t b) const
    {
        const int64_t node = kAsA ? a : b;
        const int o = int(kAsA ? b : a);
        if (node >= rows) return make_float4(0, 0, 0, 0);
        if (vec && o + 3 < Fo) {
            float4 g = *reinterpret_cast<const float4 *>(dHn + node * Fo + o);
            if (relu) {
                const float4 h = *reinterpret_cast<const float4 *>(Hn + node * Fo + o);
                g.x = h.x > 0.0f ? g.x : 0.0f;
                g.y = h.y > 0.0f ? g.y : 0.0f;
                g.z = h.z > 0.0f ? g.z : 0.0f;
                g.w = h.w > 0.0f ? g.w : 0.0f;
            }
            return g;
        }
        return make_float4(at(node, o), at(node, o + 1), at(node, o + 2), at(node, o + 3));
    }
};

// ---------------------------------------------------------------------------
// Epilogues
// ---------------------------------------------------------------------------
struct FwdEpilogue {  // H' = act(acc + b)
    float *out;
    const float *bias;
    int N;
    bool relu;
    __device__ __forceinline__ void operator()(int64_t row, int col, float v, int /*split*/) const
    {
        v += bias[col];
        if (relu) v = v > 0.0f ? v : 0.0f;
        out[row * N + col] = v;
    }
};

struct BwdDataEpilogue {  // columns [0,F): dH_self ; [F,2F): inv_deg[row] * dM
    float *dH;
    float *dMs;
    const float *inv_deg;
    int F;
    __device__ __forceinline__ void operator()(int64_t row, int col, float v, int /*split*/) const
    {
        if (col < F) dH[row * F + col] = v;
        else dMs[row * F + (col - F)] = v * inv_deg[row];
    }
};

struct SplitEpilogue {  // partial products, one slab per split
    float *partial;
    int64_t Mtot;
    int N;
    __device__ __forceinline__ void operator()(int64_t row, int col, float v, int split) const
    {
        partial[(int64_t(split) * Mtot + row) * N + col] = v;
    }
};

// ---------------------------------------------------------------------------
// C[M,N] = A[M,K] B[K,N] over k in [split*k_per_split, ...), fp32 MFMA.
// Grid: x = m-tile * n_tiles + n-tile (n fastest, so the blocks that share an
// A row block run together), y = split.
// ---------------------------------------------------------------------------
template <int BM, int BN, int BK, int WM, int WN, bool kColSum, class AL, class BL, class Epi>
__global__ __launch_bounds__(WM *WN * 64) void gemm_f32_kernel(AL a, BL b, Epi epi, int64_t M, int N, int64_t K,
                                                              int64_t k_per_split, int n_tiles,
                                                              float *__restrict__ colsum_partial)
{
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM / 32;
    constexpr int TN = BN / WN / 32;
    constexpr int A_V = BM * BK / 4 / NT;
    constexpr int B_V = BN * BK / 4 / NT;
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0 && BK % 4 == 0, "tile shape");
    static_assert((BM * BK / 4) % NT == 0 && (BN * BK / 4) % NT == 0, "loader shape");

    __shared__ __attribute__((aligned(16))) float As[BK][BM + kPad];
    __shared__ __attribute__((aligned(16))) float Bs[BK][BN + kPad];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm0 = (wave / WN) * (BM / WM);
    const int wn0 = (wave % WN) * (BN / WN);
    const int64_t m0 = int64_t(blockIdx.x / n_tiles) * BM;
    const int n0 = int(blockIdx.x % n_tiles) * BN;
    const int split = blockIdx.y;
    const int64_t k_begin = int64_t(split) * k_per_split;
    int64_t k_end = k_begin + k_per_split;
    if (k_end > K) k_end = K;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    float4 areg[A_V], breg[B_V];
    float colsum = 0.0f;

    auto fetch = [&](int64_t kt) {
#pragma unroll
        for (int i = 0; i < A_V; ++i) {
            const int idx = tid + i * NT;
            if (AL::kContigK) areg[i] = a.load4(m0 + idx / (BK / 4), kt + (idx % (BK / 4)) * 4);
            else areg[i] = a.load4(m0 + (idx % (BM / 4)) * 4, kt + idx / (BM / 4));
        }
#pragma unroll
        for (int i = 0; i < B_V; ++i) {
            const int idx = tid + i * NT;
            if (BL::kContigK) breg[i] = b.load4(n0 + idx / (BK / 4), kt + (idx % (BK / 4)) * 4);
            else breg[i] = b.load4(n0 + (idx % (BN / 4)) * 4, kt + idx / (BN / 4));
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int i = 0; i < A_V; ++i) {
            const int idx = tid + i * NT;
            if (AL::kContigK) {
                const int m = idx / (BK / 4), k = (idx % (BK / 4)) * 4;
                As[k + 0][m] = areg[i].x;
                As[k + 1][m] = areg[i].y;
                As[k + 2][m] = areg[i].z;
                As[k + 3][m] = areg[i].w;
            } else {
                *reinterpret_cast<float4 *>(&As[idx / (BM / 4)][(idx % (BM / 4)) * 4]) = areg[i];
            }
        }
#pragma unroll
        for (int i = 0; i < B_V; ++i) {
            const int idx = tid + i * NT;
            if (BL::kContigK) {
                const int n = idx / (BK / 4), k = (idx % (BK / 4)) * 4;
                Bs[k + 0][n] = breg[i].x;
                Bs[k + 1][n] = breg[i].y;
                Bs[k + 2][n] = breg[i].z;
                Bs[k + 3][n] = breg[i].w;
            } else {
                *reinterpret_cast<float4 *>(&Bs[idx / (BN / 4)][(idx % (BN / 4)) * 4]) = breg[i];
            }
        }
    };

    if (k_begin < k_end) {
        fetch(k_begin);
        stage();
    }
    __syncthreads();
    for (int64_t kt = k_begin; kt < k_end; kt += BK) {
        const bool more = kt + BK < k_end;
        if (more) fetch(kt + BK);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            float af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = As[kk + (lane >> 5)][wm0 + i * 32 + (lane & 31)];
#pragma unroll
            for (int j = 0; j < TN; ++j) bf[j] = Bs[kk + (lane >> 5)][wn0 + j * 32 + (lane & 31)];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        if (kColSum && m0 == 0 && tid < BN) {
#pragma unroll
            for (int k = 0; k < BK; ++k) colsum += Bs[k][tid];
        }
        __syncthreads();
        if (more) stage();
        __syncthreads();
    }

    // MFMA 32x32 result layout: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32.
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn0 + j * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = m0 + wm0 + i * 32 + 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
                if (row < M && col < N) epi(row, col, acc[i][j][r], split);
            }
        }
    if (kColSum && m0 == 0 && tid < BN && n0 + tid < N) colsum_partial[int64_t(split) * N + n0 + tid] = colsum;
}

// Second stage of the split reduction: fixed order over the splits.
__global__ __launch_bounds__(256) void reduce_splits_kernel(const float *__restrict__ partial,
                                                            const float *__restrict__ colsum_partial, int n_splits,
                                                            int F, int N, float *__restrict__ dW_self,
                                                            float *__restrict__ dW_neigh, float *__restrict__ dbias)
{
    const int64_t total = int64_t(2) * F * N;
    const int64_t idx = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (idx < total) {
        float s = 0.0f;
        for (int sp = 0; sp < n_splits; ++sp) s += partial[int64_t(sp) * total + idx];
        const int64_t half = int64_t(F) * N;
        if (idx < half) dW_self[idx] = s;
        else dW_neigh[idx - half] = s;
    } else if (idx < total + N) {
        const int n = int(idx - total);
        float s = 0.0f;
        for (int sp = 0; sp < n_splits; ++sp) s += colsum_partial[int64_t(sp) * N + n];
        dbias[n] = s;
    }
}

static bool vec4_ok(const void *p, int64_t ld) { return aligned(p, 16) && ld % 4 == 0; }

template <int BM, int BN, int WM, int WN, bool kColSum, class AL, class BL, class Epi>
static void launch_gemm(const char *name, const AL &a, const BL &b, const Epi &e, int64_t M, int N, int64_t K,
                        int64_t k_per_split, int n_splits, float *colsum_partial, hipStream_t s)
{
    constexpr int BK = 16;
    TMA_TIMED(name, s);
    const int n_tiles = int(ceil_div(N, BN));
    const int64_t m_tiles = ceil_div(M, BM);
    hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, BK, WM, WN, kColSum, AL, BL, Epi>),
                       dim3(unsigned(m_tiles * n_tiles), unsigned(n_splits)), dim3(WM * WN * 64), 0, s, a, b, e, M, N,
                       K, k_per_split, n_tiles, colsum_partial);
}

int launch_sage_gemm_fwd(int64_t n, const void *H, int64_t ldh, const void *M, int32_t F_in, const float *W_self,
                         const float *W_neigh, const float *bias, int32_t F_out, int32_t act, int32_t dtype,
                         void *Hnext, hipStream_t stream)
{
    if (dtype != TMA_F32) return fail(TMA_ERR_UNSUPPORTED_DTYPE, "sage gemm fwd: dtype %d not built yet", dtype);
    if (n == 0 || F_out == 0) return TMA_OK;
    const float *Hf = static_cast<const float *>(H), *Mf = static_cast<const float *>(M);
    CatRows a{Hf, ldh, Mf, F_in, n, vec4_ok(Hf, ldh) && vec4_ok(Mf, F_in) && F_in % 4 == 0};
    CatWeights b{W_self, W_neigh, F_in, F_out, vec4_ok(W_self, F_out) && vec4_ok(W_neigh, F_out)};
    FwdEpilogue e{static_cast<float *>(Hnext), bias, F_out, act == TMA_ACT_RELU};
    const int64_t K = 2 * int64_t(F_in);
    const int64_t kps = round_up(size_t(K), 16);
    if (F_out <= 64) launch_gemm<128, 64, 4, 1, false>("gemm_fwd_128x64", a, b, e, n, F_out, K, kps, 1, nullptr, stream);
    else launch_gemm<128, 128, 2, 2, false>("gemm_fwd_128x128", a, b, e, n, F_out, K, kps, 1, nullptr, stream);
    return check_launch("sage gemm fwd");
}

int launch_sage_gemm_bwd_data(int64_t n, const void *dHnext, const void *Hnext, const float *inv_deg,
                              const float *W_self, const float *W_neigh, int32_t F_in, int32_t F_out, int32_t act,
                              int32_t dtype, void *dH_self_out, void *dM_scaled_out, hipStream_t stream)
{
    if (dtype != TMA_F32) return fail(TMA_ERR_UNSUPPORTED_DTYPE, "sage gemm bwd: dtype %d not built yet", dtype);
    if (n == 0 || F_in == 0) return TMA_OK;
    const float *g = static_cast<const float *>(dHnext), *h = static_cast<const float *>(Hnext);
    const bool relu = act == TMA_ACT_RELU;
    MaskedGrad<true> a{g, h, F_out, n, relu, vec4_ok(g, F_out) && (!relu || vec4_ok(h, F_out))};
    CatWeightsT b{W_self, W_neigh, F_in, F_out, vec4_ok(W_self, F_out) && vec4_ok(W_neigh, F_out)};
    BwdDataEpilogue e{static_cast<float *>(dH_self_out), static_cast<float *>(dM_scaled_out), inv_deg, F_in};
    const int N = 2 * F_in;
    const int64_t K = F_out;
    const int64_t kps = round_up(size_t(K), 16);
    launch_gemm<128, 128, 2, 2, false>("gemm_bwd_data_128x128", a, b, e, n, N, K, kps, 1, nullptr, stream);
    return check_launch("sage gemm bwd data");
}

struct WeightSplit {
    int n_splits;
    int64_t k_per_split;
    size_t partial_bytes, colsum_bytes;
};

static WeightSplit plan_weight_split(int64_t n, int32_t F_in, int32_t F_out)
{
    const int bn = F_out <= 64 ? 64 : 128;
    const int64_t tiles = ceil_div(2 * int64_t(F_in), 128) * ceil_div(F_out, bn);
    int64_t want = ceil_div(512, tiles > 0 ? tiles : 1);
    const int64_t max_useful = ceil_div(n > 0 ? n : 1, 64);
    if (want > max_useful) want = max_useful;
    if (want < 1) want = 1;
    WeightSplit w;
    w.k_per_split = int64_t(round_up(size_t(ceil_div(n > 0 ? n : 1, want)), 16));
    w.n_splits = int(ceil_div(n > 0 ? n : 1, w.k_per_split));
    w.partial_bytes = round_up(size_t(w.n_splits) * 2 * size_t(F_in) * size_t(F_out) * 4, 256);
    w.colsum_bytes = round_up(size_t(w.n_splits) * size_t(F_out) * 4, 256);
    return w;
}

size_t sage_gemm_bwd_weight_workspace_bytes(int64_t n, int32_t F_in, int32_t F_out)
{
    const WeightSplit w = plan_weight_split(n, F_in, F_out);
    return w.partial_bytes + w.colsum_bytes;
}

int launch_sage_gemm_bwd_weight(int64_t n, const void *H, int64_t ldh, const void *M, const void *dHnext,
                                const void *Hnext, int32_t F_in, int32_t F_out, int32_t act, int32_t dtype,
                                float *dW_self, float *dW_neigh, float *dbias, void *ws, size_t ws_bytes,
                                hipStream_t stream)
{
    if (dtype != TMA_F32) return fail(TMA_ERR_UNSUPPORTED_DTYPE, "sage gemm bwd: dtype %d not built yet", dtype);
    if (F_out == 0) return TMA_OK;
    const WeightSplit w = plan_weight_split(n, F_in, F_out);
    if (ws_bytes < w.partial_bytes + w.colsum_bytes)
        return fail(TMA_ERR_WORKSPACE_TOO_SMALL, "sage gemm bwd weight: workspace %zu < %zu", ws_bytes,
                    w.partial_bytes + w.colsum_bytes);
    float *partial = static_cast<float *>(ws);
    float *colsum = reinterpret_cast<float *>(static_cast<char *>(ws) + w.partial_bytes);
    const float *Hf = static_cast<const float *>(H), *Mf = static_cast<const float *>(M);
    const float *g = static_cast<const float *>(dHnext), *h = static_cast<const float *>(Hnext);
    const bool relu = act == TMA_ACT_RELU;
    CatRowsT a{Hf, ldh, Mf, F_in, n, vec4_ok(Hf, ldh) && vec4_ok(Mf, F_in) && F_in % 4 == 0};
    MaskedGrad<false> b{g, h, F_out, n, relu, vec4_ok(g, F_out) && (!relu || vec4_ok(h, F_out))};
    const int64_t Mtot = 2 * int64_t(F_in);
    SplitEpilogue e{partial, Mtot, F_out};
    if (F_in > 0) {
        if (F_out <= 64) launch_gemm<128, 64, 4, 1, true>("gemm_bwd_weight_128x64", a, b, e, Mtot, F_out, n, w.k_per_split, w.n_splits, colsum, stream);
        else launch_gemm<128, 128, 2, 2, true>("gemm_bwd_weight_128x128", a, b, e, Mtot, F_out, n, w.k_per_split, w.n_splits, colsum, stream);
        if (int rc = check_launch("sage gemm bwd weight")) return rc;
    }
    const int64_t total = Mtot * F_out + F_out;
    TMA_TIMED("reduce_splits", stream);
    hipLaunchKernelGGL(reduce_splits_kernel, dim3(unsigned(ceil_div(total, 256))), dim3(256), 0, stream, partial,
                       colsum, F_in > 0 ? w.n_splits : 0, F_in, F_out, dW_self, dW_neigh, dbias);
    return check_launch("sage gemm bwd weight reduce");
}

}  // namespace tma
