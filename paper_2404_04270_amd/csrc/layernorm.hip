// Feature normalization of the pooled vectors (section 3.5 of the paper: a
// LayerNorm layer brings every sparse vector to zero mean and unit variance),
// forward and backward.
//
// Both directions are bound by HBM: the forward pass reads x and writes y, the
// backward pass reads dy and x and writes dx (12 bytes per element; the
// statistics and the parameters are noise).  A group of G lanes owns a vector
// and keeps it in registers (one f4 per lane for dim <= 256, up to four for
// dim = 1024), so every element is read once; means are reduced with wavefront
// shuffles, the variance from the centred values (two passes over registers,
// not the E[x^2] - mu^2 form).  The backward pass recomputes x-hat from x, mean
// and rstd instead of storing it.  The parameter gradients are sums over the
// batch: each workgroup adds up its vectors column by column in a fixed order
// and writes one partial row; a second kernel adds the partial rows in index
// order, so dgamma and dbeta do not depend on scheduling.
//
// Both kernels also come in a form that pools the vector from the tables on the
// fly (the sum of the bag's rows, in bag order, exactly as ss_embbag_forward
// forms it) instead of reading it from memory: the pooled tensor is then never
// written nor read, which at 26 x 8192 x 64 takes 109 MB out of the 273 MB the
// two passes move.
#include "ss_common.h"

namespace ss {
namespace {

// P below = f4 per lane: 1 for dim <= 256, up to 4 for dim = 64 lanes * 4 * 4 = 1024
constexpr int kLnTiles = 8;          // vectors per group and workgroup (backward)

template <int G>
__device__ __forceinline__ float group_sum(float v)
{
#pragma unroll
    for (int off = G / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, G);
    return v;
}

__device__ __forceinline__ float hsum(f4 v) { return (v.x + v.y) + (v.z + v.w); }

// loads the lane's share of a vector; lanes / slots past the row read nothing
template <int G, int P>
__device__ __forceinline__ void load_row(const f4 *__restrict__ p, int c, int D4, f4 (&v)[P])
{
#pragma unroll
    for (int i = 0; i < P; ++i) {
        const int col = c + i * G;
        v[i] = f4{0.f, 0.f, 0.f, 0.f};
        if (col < D4) v[i] = p[col];
    }
}

// Where a vector comes from: memory (x != nullptr), or the bag of rows it is the
// sum of.
struct XSource {
    const float *x;                  // [T][Bcap][dim]
    const float *const *weights;     // tables
    const int32_t *idx;              // [T][Bcap][L]
    int L;
};

// v = sum over the bag of W_t[idx[t][j][l]][:], rows added in bag order; four
// row loads are in flight at a time.
template <int G, int P>
__device__ __forceinline__ void pool_row(const XSource &src, int t, int64_t vec, int c, int D4,
                                         f4 (&v)[P])
{
    const auto W = as_global(reinterpret_cast<const f4 *>(src.weights[t]));
    const int32_t *__restrict__ ip = src.idx + vec * src.L;
    constexpr int U = 4;
#pragma unroll
    for (int i = 0; i < P; ++i) v[i] = f4{0.f, 0.f, 0.f, 0.f};
    for (int l0 = 0; l0 < src.L; l0 += U) {
        int32_t r[U];
        f4 w[U][P];
#pragma unroll
        for (int u = 0; u < U; ++u) r[u] = ip[l0 + u < src.L ? l0 + u : l0];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int i = 0; i < P; ++i) {
                const int col = c + i * G;
                w[u][i] = W[(int64_t)r[u] * D4 + (col < D4 ? col : 0)];
            }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (l0 + u < src.L) {
#pragma unroll
                for (int i = 0; i < P; ++i) v[i] = (l0 + u == 0) ? w[u][i] : v[i] + w[u][i];
            }
    }
    // lanes and slots past the row loaded column 0 to stay in bounds: they hold zeros,
    // as after load_row
#pragma unroll
    for (int i = 0; i < P; ++i)
        if (c + i * G >= D4) v[i] = f4{0.f, 0.f, 0.f, 0.f};
}

template <int G, int P, bool POOL>
__device__ __forceinline__ void fetch_x(const XSource &src, int t, int64_t vec, int c, int D4,
                                        f4 (&v)[P])
{
    if (POOL)
        pool_row<G, P>(src, t, vec, c, D4, v);
    else
        load_row<G, P>(reinterpret_cast<const f4 *>(src.x) + vec * D4, c, D4, v);
}

// A group takes V vectors of its tile (V = 4 while a vector is one f4 per lane):
// all their loads are issued before the first of them is normalised, which is
// what a pass that only streams needs most.
template <int G, int P, bool POOL>
__global__ __launch_bounds__(kWG) void ln_forward_kernel(
    XSource src, int Bcap, const int32_t *__restrict__ n_valid,
    const float *__restrict__ gamma, const float *__restrict__ beta, float eps,
    float *y, float *__restrict__ mean, float *__restrict__ rstd, int D4,
    int tiles_per_table)
{
    constexpr int NG = kWG / G, V = P == 1 ? 4 : 1;
    const int t = blockIdx.x / tiles_per_table;
    const int tile = blockIdx.x - t * tiles_per_table;
    const int n = clamp_valid(n_valid, Bcap);
    const int g = threadIdx.x / G, c = threadIdx.x % G;
    const int j0 = tile * NG * V + g;         // vectors j0 + k * NG
    if (j0 >= n) return;                      // whole groups leave together
    const float inv_d = 1.0f / (float)(D4 * 4);

    f4 v[V][P];
#pragma unroll
    for (int k = 0; k < V; ++k) {
        // vectors past n_valid fetch vector j0 again (always valid) and store nothing
        const int j = j0 + k * NG < n ? j0 + k * NG : j0;
        fetch_x<G, P, POOL>(src, t, (int64_t)t * Bcap + j, c, D4, v[k]);
    }
#pragma unroll
    for (int k = 0; k < V; ++k) {
        const int j = j0 + k * NG;
        if (j >= n) break;
        const int64_t vec = (int64_t)t * Bcap + j;
        f4 *yp = reinterpret_cast<f4 *>(y) + vec * D4;       // may be x's own row
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < P; ++i) s += hsum(v[k][i]);
        const float mu = group_sum<G>(s) * inv_d;
        float q = 0.f;
#pragma unroll
        for (int i = 0; i < P; ++i) {
            if (c + i * G < D4) {
                v[k][i] = v[k][i] - mu;
                q += hsum(v[k][i] * v[k][i]);
            }
        }
        const float var = group_sum<G>(q) * inv_d;
        const float rs = 1.0f / sqrtf(var + eps);
#pragma unroll
        for (int i = 0; i < P; ++i) {
            const int col = c + i * G;
            if (col < D4) {
                f4 o = v[k][i] * rs;
                if (gamma) o = o * reinterpret_cast<const f4 *>(gamma)[(int64_t)t * D4 + col];
                if (beta) o = o + reinterpret_cast<const f4 *>(beta)[(int64_t)t * D4 + col];
                yp[col] = o;
            }
        }
        if (c == 0) {
            mean[vec] = mu;
            rstd[vec] = rs;
        }
    }
}

// Workgroup b of a table takes vectors [b * NG * kLnTiles, (b+1) * NG * kLnTiles);
// group g takes every NG-th of them.  Partial parameter gradients: one row of
// dim floats per workgroup for dgamma and one for dbeta.
template <int G, int P, bool POOL>
__global__ __launch_bounds__(kWG) void ln_backward_kernel(
    const float *dy, XSource src, int Bcap,
    const int32_t *__restrict__ n_valid, const float *__restrict__ gamma,
    const float *__restrict__ mean, const float *__restrict__ rstd, float *dx, int D4,
    int wgs_per_table, f4 *__restrict__ part_dgamma, f4 *__restrict__ part_dbeta)
{
    constexpr int NG = kWG / G;
    __shared__ f4 s_red[kWG];
    const int t = blockIdx.x / wgs_per_table;
    const int wg = blockIdx.x - t * wgs_per_table;
    const int n = clamp_valid(n_valid, Bcap);
    const int g = threadIdx.x / G, c = threadIdx.x % G;
    const float inv_d = 1.0f / (float)(D4 * 4);
    const bool want_params = part_dgamma != nullptr;

    f4 gam[P], acc_g[P], acc_b[P];
#pragma unroll
    for (int i = 0; i < P; ++i) {
        const int col = c + i * G;
        gam[i] = f4{1.f, 1.f, 1.f, 1.f};
        if (gamma && col < D4)
            gam[i] = reinterpret_cast<const f4 *>(gamma)[(int64_t)t * D4 + col];
        acc_g[i] = acc_b[i] = f4{0.f, 0.f, 0.f, 0.f};
    }

    for (int k = 0; k < kLnTiles; ++k) {
        const int j = (wg * kLnTiles + k) * NG + g;
        if (j >= n) break;                    // later vectors of this group are past n too
        const int64_t vec = (int64_t)t * Bcap + j;
        f4 xv[P], dv[P];
        load_row<G, P>(reinterpret_cast<const f4 *>(dy) + vec * D4, c, D4, dv);
        fetch_x<G, P, POOL>(src, t, vec, c, D4, xv);
        const float mu = mean[vec], rs = rstd[vec];
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int i = 0; i < P; ++i) {
            if (c + i * G < D4) {
                xv[i] = (xv[i] - mu) * rs;                 // x-hat
                const f4 gd = gam[i] * dv[i];
                s1 += hsum(gd);
                s2 += hsum(gd * xv[i]);
                acc_g[i] = acc_g[i] + dv[i] * xv[i];
                acc_b[i] = acc_b[i] + dv[i];
            }
        }
        const float m1 = group_sum<G>(s1) * inv_d;
        const float m2 = group_sum<G>(s2) * inv_d;
        f4 *op = reinterpret_cast<f4 *>(dx) + vec * D4;      // may be dy's own row
#pragma unroll
        for (int i = 0; i < P; ++i) {
            const int col = c + i * G;
            if (col < D4) op[col] = (gam[i] * dv[i] - m1 - xv[i] * m2) * rs;
        }
    }

    if (!want_params) return;
    // column sums over the NG groups, in group order
    const int64_t prow = ((int64_t)t * wgs_per_table + wg) * D4;
#pragma unroll
    for (int i = 0; i < P; ++i) {
        const int col = c + i * G;
        for (int which = 0; which < 2; ++which) {
            s_red[threadIdx.x] = which == 0 ? acc_g[i] : acc_b[i];
            __syncthreads();
            if (g == 0 && col < D4) {
                f4 tot = s_red[c];
                for (int q = 1; q < NG; ++q) tot = tot + s_red[q * G + c];
                (which == 0 ? part_dgamma : part_dbeta)[prow + col] = tot;
            }
            __syncthreads();
        }
    }
}

// out[t][:] = sum over the workgroups' partial rows.  One workgroup per table and
// f4 column block: thread (part, col) adds every kParts-th partial row starting at
// `part`, then the kParts sums of a column are added in part order; the order is
// fixed by the shape alone.
constexpr int kRedCols = 16;                 // f4 columns per workgroup
constexpr int kParts = kWG / kRedCols;       // 16 partial sums per column

__global__ __launch_bounds__(kWG) void ln_param_reduce_kernel(
    const f4 *__restrict__ part_dgamma, const f4 *__restrict__ part_dbeta,
    int wgs_per_table, int D4, float *__restrict__ dgamma, float *__restrict__ dbeta)
{
    __shared__ f4 s_g[kWG], s_b[kWG];
    const int t = blockIdx.y;
    const int part = threadIdx.x / kRedCols;
    const int col = blockIdx.x * kRedCols + threadIdx.x % kRedCols;
    f4 sg = f4{0.f, 0.f, 0.f, 0.f}, sb = sg;
    if (col < D4) {
        const f4 *__restrict__ pg = part_dgamma + (int64_t)t * wgs_per_table * D4 + col;
        const f4 *__restrict__ pb = part_dbeta + (int64_t)t * wgs_per_table * D4 + col;
        for (int w = part; w < wgs_per_table; w += kParts) {
            sg = sg + pg[(int64_t)w * D4];
            sb = sb + pb[(int64_t)w * D4];
        }
    }
    s_g[threadIdx.x] = sg;
    s_b[threadIdx.x] = sb;
    __syncthreads();
    if (part == 0 && col < D4) {
        for (int q = 1; q < kParts; ++q) {
            sg = sg + s_g[q * kRedCols + threadIdx.x];
            sb = sb + s_b[q * kRedCols + threadIdx.x];
        }
        if (dgamma) reinterpret_cast<f4 *>(dgamma)[(int64_t)t * D4 + col] = sg;
        if (dbeta) reinterpret_cast<f4 *>(dbeta)[(int64_t)t * D4 + col] = sb;
    }
}

int backward_wgs(int dim, int Bcap)
{
    const int per_wg = (kWG / lanes_per_row(dim)) * kLnTiles;
    return (Bcap + per_wg - 1) / per_wg;
}

}  // namespace

int32_t launch_layernorm_forward(int T, int dim, const float *x, const float *const *weights,
                                 const int32_t *idx, int L, int Bcap, const int32_t *n_valid,
                                 const float *gamma, const float *beta, float eps, float *y,
                                 float *mean, float *rstd, hipStream_t s)
{
    const XSource src{x, weights, idx, L};
    const int D4 = dim / 4, g = lanes_per_row(dim);
    const int per_tile = (kWG / g) * (D4 <= g ? 4 : 1);      // as V in the kernel
    const int tiles = (Bcap + per_tile - 1) / per_tile;
    if ((int64_t)tiles * T > 0x7fffffffLL)
        return fail(SS_ERR_UNSUPPORTED, "ss_layernorm_forward: grid too large");
    ProfScope prof(x ? "ln_forward_kernel" : "ln_forward_pool_kernel", s);
#define SS_LN_FWD(P_)                                                                   \
    if (x)                                                                              \
        launch(ln_forward_kernel<G, P_, false>, dim3((unsigned)(tiles * T)), dim3(kWG), s, \
               src, Bcap, n_valid, gamma, beta, eps, y, mean, rstd, D4, tiles);         \
    else                                                                                \
        launch(ln_forward_kernel<G, P_, true>, dim3((unsigned)(tiles * T)), dim3(kWG), s, \
               src, Bcap, n_valid, gamma, beta, eps, y, mean, rstd, D4, tiles)
    SS_DISPATCH_G(g, if constexpr (G < 64) { SS_LN_FWD(1); } else {
        if (D4 <= 64) { SS_LN_FWD(1); } else if (D4 <= 128) { SS_LN_FWD(2); } else { SS_LN_FWD(4); }
    });
#undef SS_LN_FWD
    return check_launch("ss_layernorm_forward");
}

size_t layernorm_backward_ws_bytes(int T, int dim, int Bcap)
{
    return align_up((size_t)2 * T * backward_wgs(dim, Bcap) * dim * sizeof(float), 256);
}

int32_t launch_layernorm_backward(int T, int dim, const float *dy, const float *x,
                                  const float *const *weights, const int32_t *idx, int L,
                                  int Bcap, const int32_t *n_valid, const float *gamma,
                                  const float *mean, const float *rstd, float *dx,
                                  float *dgamma, float *dbeta, void *ws, hipStream_t s)
{
    const XSource src{x, weights, idx, L};
    const int D4 = dim / 4, g = lanes_per_row(dim);
    const int wgs = backward_wgs(dim, Bcap);
    if ((int64_t)wgs * T > 0x7fffffffLL)
        return fail(SS_ERR_UNSUPPORTED, "ss_layernorm_backward: grid too large");
    const bool params = dgamma || dbeta;
    f4 *pg = params ? static_cast<f4 *>(ws) : nullptr;
    f4 *pb = params ? pg + (size_t)T * wgs * D4 : nullptr;
    {
        ProfScope prof(x ? "ln_backward_kernel" : "ln_backward_pool_kernel", s);
#define SS_LN_BWD(P_)                                                                   \
    if (x)                                                                              \
        launch(ln_backward_kernel<G, P_, false>, dim3((unsigned)(wgs * T)), dim3(kWG), s, dy, \
               src, Bcap, n_valid, gamma, mean, rstd, dx, D4, wgs, pg, pb);             \
    else                                                                                \
        launch(ln_backward_kernel<G, P_, true>, dim3((unsigned)(wgs * T)), dim3(kWG), s, dy, \
               src, Bcap, n_valid, gamma, mean, rstd, dx, D4, wgs, pg, pb)
        SS_DISPATCH_G(g, if constexpr (G < 64) { SS_LN_BWD(1); } else {
            if (D4 <= 64) { SS_LN_BWD(1); } else if (D4 <= 128) { SS_LN_BWD(2); } else { SS_LN_BWD(4); }
        });
#undef SS_LN_BWD
    }
    if (params)
        launch(ln_param_reduce_kernel, dim3((D4 + kRedCols - 1) / kRedCols, T), dim3(kWG), s,
               (const f4 *)pg, (const f4 *)pb, wgs, D4, dgamma, dbeta);
    return check_launch("ss_layernorm_backward");
}

}  // namespace ss
