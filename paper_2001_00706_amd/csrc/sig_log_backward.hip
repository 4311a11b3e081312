// Gradient through the logarithm of signatures (the logarithm of section 2.3 as one more differentiable
// primitive, section 5.3) and through the selection of the Lyndon words (appendix A.2.4).
//
// The forward value is Horner's rule  R_N = c_N x,  R_m = c_m x + x * R_{m+1},  log = R_1  (x the signature
// without its constant term, c_m = (-1)^{m+1} / m, * the product of elements without constant terms, R_m kept
// at levels 1..N-m+1).  Its reverse, with G_m the cotangent of R_m and G_1 the incoming gradient:
//     gx       += c_m G_m
//     gx[u]    += sum_v G_m[u v] R_{m+1}[v]        (every split of a word into a prefix u and a suffix v)
//     G_{m+1}[v] = sum_u x[u] G_m[u v]
// for m = 1..N-1, and gx += c_N G_N at the end.
//
// Layout makes both sums matrix-vector products.  In a flat element the levels l+1..n of G, read from the
// offset of level l+1, ARE a row-major matrix M_l with d^l columns whose row number is the flat position of
// the prefix u (levels 1..n-l of x or gx) and whose column is the suffix v (level l).  So per step and per l:
//     a_l = x[0 .. U_l)^T M_l  -> level l of G_{m+1},        b_l = M_l R_{m+1, level l}  -> added into gx[0 .. U_l).
// One launch per step walks every M_l once, in contiguous pieces: column sums stay in the lanes, row dots are
// reduced inside a wavefront.  Pieces of one matrix go to different workgroups, which write partial sums; a
// second launch adds them up in a fixed order (no atomics: the result does not depend on scheduling).
// The R_m are recomputed first, one launch per m, into the workspace.
#include "sig_internal.h"
#include "sig_lane_ops.h"

namespace sig {
namespace {

constexpr int kLbThreads = 256;
constexpr int kLbWideRows = 16;   // rows between two workgroup barriers in a matrix with more than 256 columns
constexpr int kLbWideCols = 8;    // columns per lane there: a workgroup spans 2048 columns
constexpr uint32_t kLbMaxPartials = 32;   // partial sums per output the planner aims for
constexpr int kFusedRows = 4;             // passes the single-launch kernel forms between two barriers

struct LbLevel {               // the matrix M_l of one step
    uint32_t C;                // columns, d^l
    uint32_t U;                // rows, S(n - l)
    uint32_t base;             // where the matrix starts inside G: offset of level l + 1
    uint32_t wg_start;         // first workgroup (of those serving one batch row) that works on it
    uint32_t wide;             // 0: C <= 256, several rows per pass; 1: 2048 columns per workgroup, a row at a time
    uint32_t rows_per_wg;
    uint32_t tiles;            // column tiles (1 unless wide)
    uint32_t chunks;           // row chunks = partial column sums per column
    uint32_t rpw;              // narrow: rows per pass
    uint32_t lg_tpr;           // narrow: log2 of the lanes that share one row dot
    int64_t apart_off, bpart_off;   // where its partial sums start inside a batch row's share of the buffers
};

struct LbStep {
    int count;                 // matrices: l = 1..count, G has count + 1 levels
    uint32_t wgs;              // workgroups per batch row
    uint32_t S_next, S_cur;    // S(n - 1), S(n)
    int64_t apart_stride, bpart_stride;   // per batch row
    LbLevel lv[SIG_MAX_DEPTH];
};

template <typename T>
__device__ __forceinline__ T lanes_sum(T s, uint32_t lg)   // sum over aligned groups of 2^lg lanes (lg <= 6)
{
    switch (lg) {
        case 1: return group_sum<0, 1, T>(s);
        case 2: return group_sum<0, 2, T>(s);
        case 3: return group_sum<0, 3, T>(s);
        case 4: return group_sum<0, 4, T>(s);
        case 5: return group_sum<0, 5, T>(s);
        case 6: return group_sum<0, 6, T>(s);
    }
    return s;
}

// R_m = c_m x + x * R_{m+1} at levels 1..n (n = N - m + 1); R_{m+1} null for m = N.  One thread per scalar.
template <typename T, int D>
__global__ void __launch_bounds__(kLbThreads)
log_bwd_horner_kernel(Shape sh, int n, T c_m, const T *__restrict__ x, const T *__restrict__ r_next, T *__restrict__ r_out,
                      int64_t r_stride)
{
    const uint32_t d = D > 0 ? uint32_t(D) : uint32_t(sh.d);
    const int64_t S_n = sh.off[n + 1];
    const int64_t gid = int64_t(blockIdx.x) * kLbThreads + threadIdx.x;
    if (gid >= sh.B * S_n) return;
    const int64_t row = gid / S_n;
    const uint32_t q = uint32_t(gid - row * S_n);
    int k = 1;
    while (k < n && q >= uint32_t(sh.off[k + 1])) ++k;
    const T *xr = x + row * sh.S;
    T acc = c_m * xr[q];
    if (r_next != nullptr) {
        const T *rr = r_next + row * r_stride;
        uint32_t prefix = q - uint32_t(sh.off[k]), suffix = 0, scale = 1;
        for (int j = k - 1; j >= 1; --j) {
            const uint32_t letter = prefix % d;
            prefix /= d;
            suffix += letter * scale;
            scale *= d;
            acc += xr[uint32_t(sh.off[j]) + prefix] * rr[uint32_t(sh.off[k - j]) + suffix];
        }
    }
    r_out[row * r_stride + q] = acc;
}

// One step: partial column sums (x^T M_l) and row dots (M_l R_l) of every matrix of the step.
template <typename T>
__global__ void __launch_bounds__(kLbThreads)
log_bwd_main_kernel(LbStep stp, const T *__restrict__ x, int64_t x_stride, int64_t x_group, const T *__restrict__ G,
                    int64_t g_stride, const T *__restrict__ R, int64_t r_stride, T *__restrict__ apart, T *__restrict__ bpart)
{
    __shared__ T prod[2][kLbThreads];
    __shared__ T wsum[kLbWideRows][kLbThreads / 64];
    const uint32_t tid = threadIdx.x;
    const uint32_t wg = blockIdx.x % stp.wgs;
    const int64_t row = blockIdx.x / stp.wgs;
    int li = 0;
    for (int i = 1; i < stp.count; ++i)
        if (wg >= stp.lv[i].wg_start) li = i;
    const LbLevel lv = stp.lv[li];
    const uint32_t C = lv.C, U = lv.U;
    const T *xr = x + (row / x_group) * x_stride;   // x_group consecutive rows share one left factor
    const T *M = G + row * g_stride + lv.base;
    const T *Rl = R + row * r_stride + (lv.base - C);   // level l of R_{m+1}
    T *ap = apart + row * stp.apart_stride + lv.apart_off;
    T *bp = bpart + row * stp.bpart_stride + lv.bpart_off;
    const uint32_t w = wg - lv.wg_start;

    if (lv.wide == 0) {
        const uint32_t rpw = lv.rpw;
        const bool on = tid < rpw * C;
        const uint32_t prow = on ? tid / C : 0, col = on ? tid - prow * C : 0;
        const T rl = on ? Rl[col] : T(0);
        const uint32_t row0 = w * lv.rows_per_wg;
        const uint32_t row_end = row0 + lv.rows_per_wg < U ? row0 + lv.rows_per_wg : U;
        const uint32_t tpr = 1u << lv.lg_tpr;
        const uint32_t srow = tid >> lv.lg_tpr, sub = tid & (tpr - 1);
        T acc = T(0);
        int buf = 0;
        for (uint32_t r = row0; r < row_end; r += rpw, buf ^= 1) {
            const uint32_t mine = r + prow;
            T g = T(0);
            if (on && mine < row_end) {
                g = M[uint64_t(mine) * C + col];
                acc += xr[mine] * g;
            }
            prod[buf][tid] = g * rl;
            __syncthreads();
            // row dots: 2^lg_tpr lanes per row, each over a strided share of the row's products
            T s = T(0);
            if (srow < rpw)
                for (uint32_t c = sub; c < C; c += tpr) s += prod[buf][srow * C + c];
            s = lanes_sum(s, lv.lg_tpr);
            if (sub == 0 && srow < rpw && r + srow < row_end) bp[r + srow] = s;
        }
        // column sums: fold the rows of a pass
        __syncthreads();
        prod[0][tid] = acc;
        __syncthreads();
        if (tid < C) {
            T s = T(0);
            for (uint32_t p = 0; p < rpw; ++p) s += prod[0][p * C + tid];
            ap[uint64_t(w) * C + tid] = s;
        }
    } else {
        const uint32_t tile = w % lv.tiles, chunk = w / lv.tiles;
        const uint32_t col0 = tile * (kLbThreads * kLbWideCols) + tid;   // this lane's columns: col0 + 256 v
        T rl[kLbWideCols], acc[kLbWideCols];
#pragma unroll
        for (int v = 0; v < kLbWideCols; ++v) {
            const uint32_t col = col0 + v * kLbThreads;
            rl[v] = col < C ? Rl[col] : T(0);
            acc[v] = T(0);
        }
        const uint32_t row0 = chunk * lv.rows_per_wg;
        const uint32_t row_end = row0 + lv.rows_per_wg < U ? row0 + lv.rows_per_wg : U;
        for (uint32_t rb = row0; rb < row_end; rb += kLbWideRows) {
            const uint32_t rb_end = rb + kLbWideRows < row_end ? rb + kLbWideRows : row_end;
            for (uint32_t r = rb; r < rb_end; ++r) {
                const T *mrow = M + uint64_t(r) * C;
                const T xv = xr[r];
                T s = T(0);
#pragma unroll
                for (int v = 0; v < kLbWideCols; ++v) {
                    const uint32_t col = col0 + v * kLbThreads;
                    const T g = col < C ? mrow[col] : T(0);
                    acc[v] += xv * g;
                    s += g * rl[v];
                }
                s = group_sum<0, 6, T>(s);
                if ((tid & 63) == 0) wsum[r - rb][tid >> 6] = s;
            }
            __syncthreads();
            if (tid < rb_end - rb) {
                T s = wsum[tid][0];
                for (int v = 1; v < kLbThreads / 64; ++v) s += wsum[tid][v];
                bp[uint64_t(tile) * U + rb + tid] = s;
            }
            __syncthreads();
        }
#pragma unroll
        for (int v = 0; v < kLbWideCols; ++v) {
            const uint32_t col = col0 + v * kLbThreads;
            if (col < C) ap[uint64_t(chunk) * C + col] = acc[v];
        }
    }
}

// Adds the partial sums of a step: G_{m+1} (unless this is the last step) and gx.
//   first: gx is written, not added to.   last: G_{m+1} = G_N has one level and goes straight into gx with c_N.
//   plus_g: the column sums are the gradient of the right factor of a group product, whose unit term adds G
//           itself at every level (G_next then has as many levels as G).
template <typename T>
__global__ void __launch_bounds__(kLbThreads)
log_bwd_finish_kernel(LbStep stp, int64_t rows, T c_m, T c_last, int first, int last, int plus_g, const T *__restrict__ G,
                      int64_t g_stride, const T *__restrict__ apart, const T *__restrict__ bpart, T *__restrict__ G_next,
                      int64_t gn_stride, T *__restrict__ gx, int64_t gx_stride)
{
    const int64_t per_row = int64_t(stp.S_next) + stp.S_cur + (plus_g ? stp.S_cur - stp.S_next : 0);
    const int64_t gid = int64_t(blockIdx.x) * kLbThreads + threadIdx.x;
    if (gid >= rows * per_row) return;
    const int64_t row = gid / per_row;
    const uint32_t q = uint32_t(gid - row * per_row);
    const T *ap = apart + row * stp.apart_stride;
    const T *bp = bpart + row * stp.bpart_stride;
    if (q < stp.S_next) {
        if (last) return;
        int li = 0;   // the level of G_{m+1} this scalar lies in: offset of level l = base_l - C_l
        for (int i = 1; i < stp.count; ++i)
            if (q >= stp.lv[i].base - stp.lv[i].C) li = i;
        const LbLevel lv = stp.lv[li];
        const uint32_t v = q - (lv.base - lv.C);
        const T *p = ap + lv.apart_off + v;
        T s = T(0);
#pragma unroll 8
        for (uint32_t k = 0; k < lv.chunks; ++k) s += p[uint64_t(k) * lv.C];
        if (plus_g) s += G[row * g_stride + q];
        G_next[row * gn_stride + q] = s;
        return;
    }
    if (q >= stp.S_next + stp.S_cur) {   // plus_g: the top level of G_next is that of G
        const uint32_t top = q - stp.S_cur;
        G_next[row * gn_stride + top] = G[row * g_stride + top];
        return;
    }
    const uint32_t rho = q - stp.S_next;
    T val = c_m * G[row * g_stride + rho];
    if (!first) val += gx[row * gx_stride + rho];
    for (int i = 0; i < stp.count; ++i) {
        const uint32_t U = stp.lv[i].U;
        if (rho >= U) break;   // U shrinks as l grows
        const T *p = bp + stp.lv[i].bpart_off + rho;
        const uint32_t tiles = stp.lv[i].tiles;
#pragma unroll 8
        for (uint32_t t = 0; t < tiles; ++t) val += p[uint64_t(t) * U];
    }
    if (last && rho < stp.lv[0].C) {
        const T *p = ap + stp.lv[0].apart_off + rho;
        T s = T(0);
        for (uint32_t k = 0; k < stp.lv[0].chunks; ++k) s += p[uint64_t(k) * stp.lv[0].C];
        val += c_last * s;
    }
    gx[row * gx_stride + rho] = val;
}

// Everything above in one launch for signatures small enough to live in LDS: one workgroup per signature keeps x,
// the R_m, two cotangent buffers and the gradient on chip and walks the same matrices M_l, a whole matrix at a
// time, so that column sums stay in registers (or, beyond 256 columns, in LDS) and row dots are added straight
// into the gradient: no partial sums, no second kernel, no workspace.  A barrier separates the matrices of a
// step (they all add into the first rows of the gradient).
// The incoming gradient G_1 is read from global memory (staging it in LDS as well changed nothing), kFusedRows
// passes are formed between two barriers.
//   LDS layout (scalars): x[S] | R_N .. R_2 [r_stride] | G[2][S(N-1)] (G_2, G_3, ..) | gx[S] |
//                         prod[2][kFusedRows][NT] | wsum[NT / 64]
// NT = 256 threads for the smallest signatures (several workgroups per compute unit), 1024 beyond 2048 scalars,
// where one signature fills the LDS of a compute unit anyway and four wavefronts per SIMD issue faster than one.
template <typename T, int NT>
__global__ void __launch_bounds__(NT)
log_bwd_fused_kernel(Shape sh, int64_t r_stride, const T *__restrict__ x_g, const T *__restrict__ g_g, T *__restrict__ gx_g)
{
    extern __shared__ __align__(16) unsigned char lb_smem[];
    __shared__ uint32_t off[SIG_MAX_DEPTH + 2], pw[SIG_MAX_DEPTH + 1];
    const int N = sh.N;
    const uint32_t tid = threadIdx.x;
    const uint32_t d = uint32_t(sh.d), S = uint32_t(sh.S);
    if (tid <= uint32_t(N) + 1) off[tid] = uint32_t(sh.off[tid]);
    if (tid <= uint32_t(N)) pw[tid] = uint32_t(sh.pw[tid]);
    __syncthreads();
    const uint32_t S_low = off[N];   // S(N - 1)
    T *xs = reinterpret_cast<T *>(lb_smem);
    T *Rs = xs + S;
    T *Gb[2] = {Rs + r_stride, Rs + r_stride + S_low};   // Gb[m & 1] holds G_m, m >= 2
    T *gxs = Gb[1] + S_low;
    T *prod = gxs + S;               // [2][256]
    T *wsum = prod + 2 * kFusedRows * NT;  // [NT / 64]
    auto coef = [](int m) { return (m & 1 ? T(1) : T(-1)) / T(m); };
    auto r_at = [&](int m) {   // R_m inside Rs: R_N first
        uint32_t o = 0;
        for (int mm = N; mm > m; --mm) o += off[N - mm + 2];
        return Rs + o;
    };

    for (int64_t row = blockIdx.x; row < sh.B; row += gridDim.x) {
        const T *g_row = g_g + row * S;
        __syncthreads();   // the previous signature's gradient has been written out
        for (uint32_t i = tid; i < S; i += NT) xs[i] = x_g[row * S + i];
        __syncthreads();
        // R_m = c_m x + x * R_{m+1}, levels 1..N-m+1
        for (int m = N; m >= 2; --m) {
            const int n = N - m + 1;
            const T c = coef(m);
            T *r_out = r_at(m);
            const T *r_next = m == N ? nullptr : r_at(m + 1);
            for (uint32_t q = tid; q < off[n + 1]; q += NT) {
                int k = 1;
                while (k < n && q >= off[k + 1]) ++k;
                T acc = c * xs[q];
                if (r_next != nullptr) {
                    uint32_t prefix = q - off[k], suffix = 0, scale = 1;
                    for (int j = k - 1; j >= 1; --j) {
                        const uint32_t letter = prefix % d;
                        prefix /= d;
                        suffix += letter * scale;
                        scale *= d;
                        acc += xs[off[j] + prefix] * r_next[off[k - j] + suffix];
                    }
                }
                r_out[q] = acc;
            }
            __syncthreads();
        }
        for (int m = 1; m <= N - 1; ++m) {
            const int n = N - m + 1;
            const T *G = m == 1 ? g_row : Gb[m & 1];
            T *Gn = Gb[(m + 1) & 1];
            const T *R = r_at(m + 1);
            const T c = coef(m);
            for (uint32_t q = tid; q < off[n + 1]; q += NT) gxs[q] = (m == 1 ? T(0) : gxs[q]) + c * G[q];
            __syncthreads();
            for (int l = 1; l <= n - 1; ++l) {
                const uint32_t C = pw[l], U = off[n - l + 1];
                const T *M = G + off[l + 1];
                const T *Rl = R + off[l];
                T *Gl = Gn + off[l];
                if (C <= uint32_t(NT)) {
                    const uint32_t rpw = uint32_t(NT) / C;
                    uint32_t tpr = uint32_t(NT) / rpw, lg = 0;
                    tpr = tpr > 64 ? 64 : tpr;
                    while ((2u << lg) <= tpr) ++lg;
                    tpr = 1u << lg;
                    const bool on = tid < rpw * C;
                    const uint32_t prow = on ? tid / C : 0, col = on ? tid - prow * C : 0;
                    const T rl = on ? Rl[col] : T(0);
                    const uint32_t srow = tid >> lg, sub = tid & (tpr - 1);
                    T acc = T(0);
                    // pass r: products of rpw rows into prod[buf]; barrier; row sums out of prod[buf] into gx.  The
                    // products of the next pass are formed before the sums of this one are taken, so that the two
                    // chains of LDS round trips overlap.
                    auto form = [&](uint32_t r, int buf) {
#pragma unroll
                        for (int v = 0; v < kFusedRows; ++v) {
                            const uint32_t mine = r + v * rpw + prow;
                            T g = T(0);
                            if (on && mine < U) {
                                g = M[mine * C + col];
                                acc += xs[mine] * g;
                            }
                            prod[(buf * kFusedRows + v) * NT + tid] = g * rl;
                        }
                    };
                    form(0, 0);
                    int buf = 0;
                    for (uint32_t r = 0; r < U; r += kFusedRows * rpw, buf ^= 1) {
                        __syncthreads();
                        if (r + kFusedRows * rpw < U) form(r + kFusedRows * rpw, buf ^ 1);
#pragma unroll
                        for (int v = 0; v < kFusedRows; ++v) {
                            const uint32_t r_v = r + v * rpw;
                            if (r_v >= U) break;   // the same for every thread
                            const T *pv = prod + (buf * kFusedRows + v) * NT;
                            T t = T(0);
                            if (srow < rpw)
                                for (uint32_t cc = sub; cc < C; cc += tpr) t += pv[srow * C + cc];
                            t = lanes_sum(t, lg);
                            if (sub == 0 && srow < rpw && r_v + srow < U) gxs[r_v + srow] += t;
                        }
                    }
                    // column sums: the rpw lanes of a column are folded in two stages (up to 16 at a time, then the
                    // up to 16 group sums), never one long loop in a single thread
                    __syncthreads();
                    prod[tid] = acc;
                    __syncthreads();
                    const uint32_t groups = (rpw + 15) / 16;   // groups * C <= NT: the second half of prod holds them
                    if (tid < groups * C) {
                        const uint32_t grp = tid / C, cc = tid - grp * C;
                        T t = T(0);
#pragma unroll
                        for (uint32_t k = 0; k < 16; ++k) {   // fixed trip count: the 16 reads are in flight together
                            const uint32_t pr = grp * 16 + k;
                            t += pr < rpw ? prod[pr * C + cc] : T(0);
                        }
                        prod[NT + tid] = t;
                    }
                    __syncthreads();
                    if (tid < C) {
                        T t = T(0);
                        if (groups <= 16) {
#pragma unroll
                            for (uint32_t grp = 0; grp < 16; ++grp) t += grp < groups ? prod[NT + grp * C + tid] : T(0);
                        } else {
                            for (uint32_t grp = 0; grp < groups; ++grp) t += prod[NT + grp * C + tid];
                        }
                        Gl[tid] = t;
                    }
                } else {
                    // a row at a time, the lanes striding over its columns; column sums accumulate in LDS
                    for (uint32_t r = 0; r < U; ++r) {
                        const T xv = xs[r];
                        T part = T(0);
                        for (uint32_t col = tid; col < C; col += NT) {
                            const T g = M[r * C + col];
                            Gl[col] = (r == 0 ? T(0) : Gl[col]) + xv * g;
                            part += g * Rl[col];
                        }
                        part = group_sum<0, 6, T>(part);
                        if ((tid & 63) == 0) wsum[tid >> 6] = part;
                        __syncthreads();
                        if (tid == 0) {
                            T total = wsum[0];
                            for (int v = 1; v < NT / 64; ++v) total += wsum[v];
                            gxs[r] += total;
                        }
                        __syncthreads();
                    }
                }
                __syncthreads();
            }
        }
        // G_N has one level
        const T *G_last = Gb[N & 1];
        if (tid < d) gxs[tid] += coef(N) * G_last[tid];
        __syncthreads();
        for (uint32_t i = tid; i < S; i += NT) gx_g[row * S + i] = gxs[i];
    }
}

// The single-launch kernel for d = 2, 4, 8 written as gathers: no products parked in LDS, two barriers per step.
// Both sums of a step are dot products along the flat order of a truncated element:
//     G_{m+1}[v] = sum_t x[t] G_m[u_t v]          t runs over the flat positions of the words u_t of 1..n-|v| letters
//     gx[u]     += sum_t G_m[u v_t] R_{m+1}[t]    t runs over the flat positions of the words v_t of 1..n-|u| letters
// and the word u v of k letters sits at off_k + (u << |v| log2 d) + v.  An output of level lambda has S(n - lambda)
// terms and there are d^lambda of them, so every level holds about the same number of terms: the whole workgroup
// takes the levels one after the other, NT / d^lambda threads per output, each with every (NT / d^lambda)-th word of
// every length.  In the first sum consecutive threads hold consecutive v, in the second consecutive threads hold
// consecutive t, so that both read consecutive addresses.  The threads of an output meet by lane exchanges inside a
// wavefront and, where an output spans several wavefronts, through partial sums in LDS that are added, in a fixed
// order, after the step's first barrier.  d, N and the workgroup size are compile-time constants: every loop below
// unrolls and every offset folds (with run-time bounds the loop control was five sixths of the instructions).
// LDS: x[S] | R_N .. R_2 [r_stride] | G[2][S(N-1)] | gx[S] | partial sums.
template <int LOGD>
__host__ __device__ constexpr uint32_t gather_off(int k)   // offset of level k (1-based) in a flat element
{
    uint32_t o = 0;
    for (int j = 1; j < k; ++j) o += 1u << uint32_t(LOGD * j);
    return o;
}

template <int LOGD>
__host__ __device__ constexpr uint32_t gather_partials(int n, uint32_t nt)   // partial sums of the first kind in one step
{
    uint32_t total = 0;
    for (int lam = 1; lam <= n - 1; ++lam) {
        const uint32_t shl = uint32_t(LOGD * lam);
        if (shl >= 31 || (1u << shl) >= nt) break;
        total += (1u << shl) < 64 ? (nt >> 6) << shl : nt;
    }
    return total;
}
constexpr uint32_t kGatherPartB = 64;   // partial sums of the second kind (outputs that span several wavefronts)

template <typename T, int LOGD, int NT, int n, bool FIRST, typename GPtr>
__device__ __forceinline__ void gather_step(T c, GPtr G, T *__restrict__ Gn, const T *__restrict__ R, const T *__restrict__ xs,
                                            T *__restrict__ gxs, T *__restrict__ part, T *__restrict__ part_b, uint32_t tid)
{
    constexpr uint32_t lg_nt = NT == 1024 ? 10 : NT == 512 ? 9 : 8, waves = NT / 64;
    static_assert(NT == 1024 || NT == 512 || NT == 256, "workgroup sizes of this kernel");
    const uint32_t lane = tid & 63, wave = tid >> 6;
    // the top level of G_m reaches the gradient only through its coefficient
    for (uint32_t q = gather_off<LOGD>(n) + tid; q < gather_off<LOGD>(n + 1); q += NT) gxs[q] = (FIRST ? T(0) : gxs[q]) + c * G[q];

    // ---- every level's dot products first (all their loads are independent of one another) ...
    T acc_a[n], acc_b[n];
#pragma unroll
    for (int lam = 1; lam <= n - 1; ++lam) {
        const uint32_t shl = uint32_t(LOGD * lam);
        const int jmax = n - lam;
        acc_a[lam] = acc_b[lam] = T(0);
        if (shl >= lg_nt) {
            // at least as many outputs as threads: a thread takes whole outputs (they have few terms)
            const uint32_t outputs = 1u << shl;
            for (uint32_t v = tid; v < outputs; v += NT) {
                T acc = T(0), accb = T(0);
#pragma unroll
                for (int j = 1; j <= jmax; ++j) {
                    const uint32_t cnt = 1u << uint32_t(LOGD * j), lo = gather_off<LOGD>(j);
                    const uint32_t base_a = gather_off<LOGD>(j + lam) + v;
                    const uint32_t base_b = gather_off<LOGD>(lam + j) + (v << uint32_t(LOGD * j));
#pragma unroll 8
                    for (uint32_t p = 0; p < cnt; ++p) {
                        acc += xs[lo + p] * G[base_a + (p << shl)];
                        accb += G[base_b + p] * R[lo + p];
                    }
                }
                const uint32_t q = gather_off<LOGD>(lam) + v;
                Gn[q] = acc;
                gxs[q] = (FIRST ? T(0) : gxs[q]) + c * G[q] + accb;
            }
            continue;
        }
        const uint32_t outputs = 1u << shl, lg_tl = lg_nt - shl, tl_count = 1u << lg_tl;   // threads per output
        {   // level lambda of G_{m+1}: thread = (tl, v), v fastest
            const uint32_t v = tid & (outputs - 1), tl = tid >> shl;
#pragma unroll
            for (int j = 1; j <= jmax; ++j) {
                const uint32_t cnt = 1u << uint32_t(LOGD * j), lo = gather_off<LOGD>(j), base = gather_off<LOGD>(j + lam) + v;
                if (cnt >= tl_count) {
#pragma unroll
                    for (uint32_t k = 0; k < cnt / tl_count; ++k) {
                        const uint32_t p = tl + k * tl_count;
                        acc_a[lam] += xs[lo + p] * G[base + (p << shl)];
                    }
                } else if (tl < cnt) {
                    acc_a[lam] += xs[lo + tl] * G[base + (tl << shl)];
                }
            }
        }
        {   // gx at the words u of lambda letters: thread = (u, tl), tl fastest
            const uint32_t tl = tid & (tl_count - 1), u = tid >> lg_tl;
#pragma unroll
            for (int l = 1; l <= jmax; ++l) {
                const uint32_t cnt = 1u << uint32_t(LOGD * l), lo = gather_off<LOGD>(l);
                const uint32_t base = gather_off<LOGD>(lam + l) + (u << uint32_t(LOGD * l));
                if (cnt >= tl_count) {
#pragma unroll
                    for (uint32_t k = 0; k < cnt / tl_count; ++k) {
                        const uint32_t p = tl + k * tl_count;
                        acc_b[lam] += G[base + p] * R[lo + p];
                    }
                } else if (tl < cnt) {
                    acc_b[lam] += G[base + tl] * R[lo + tl];
                }
            }
        }
    }
    // ---- ... then the lane exchanges, one distance at a time for all levels together, so that the exchanges of the
    // levels overlap instead of forming one long chain
#pragma unroll
    for (uint32_t mask = 1; mask < 64; mask <<= 1) {
#pragma unroll
        for (int lam = 1; lam <= n - 1; ++lam) {
            const uint32_t shl = uint32_t(LOGD * lam);
            if (shl >= lg_nt) continue;
            const uint32_t outputs = 1u << shl, tl_count = 1u << (lg_nt - shl);
            if (outputs < 64 && mask >= outputs) acc_a[lam] += __shfl_xor(acc_a[lam], int(mask));
            if (mask < (tl_count < 64 ? tl_count : 64u)) acc_b[lam] += __shfl_xor(acc_b[lam], int(mask));
        }
    }
    uint32_t pbase = 0, pbase_b = 0;
#pragma unroll
    for (int lam = 1; lam <= n - 1; ++lam) {
        const uint32_t shl = uint32_t(LOGD * lam);
        if (shl >= lg_nt) continue;
        const uint32_t outputs = 1u << shl, lg_tl = lg_nt - shl, tl_count = 1u << lg_tl;
        if (outputs < 64) {
            if (lane < outputs) part[pbase + wave * outputs + lane] = acc_a[lam];
            pbase += waves << shl;
        } else {
            part[pbase + tid] = acc_a[lam];   // = [tl][v]
            pbase += NT;
        }
        const uint32_t tl = tid & (tl_count - 1), u = tid >> lg_tl;
        if (tl_count <= 64) {
            const uint32_t q = gather_off<LOGD>(lam) + u;
            if (tl == 0) gxs[q] = (FIRST ? T(0) : gxs[q]) + c * G[q] + acc_b[lam];
        } else {
            const uint32_t per = tl_count >> 6;   // wavefronts per output
            if (lane == 0) part_b[pbase_b + u * per + (wave & (per - 1))] = acc_b[lam];
            pbase_b += outputs * per;
        }
    }
    __syncthreads();
    // the partial sums, in a fixed order
    pbase = 0;
    pbase_b = 0;
#pragma unroll
    for (int lam = 1; lam <= n - 1; ++lam) {
        const uint32_t shl = uint32_t(LOGD * lam);
        if (shl >= lg_nt) break;
        const uint32_t outputs = 1u << shl, tl_count = 1u << (lg_nt - shl);
        const uint32_t count = outputs < 64 ? waves : tl_count;
        for (uint32_t v = tid; v < outputs; v += NT) {
            T total = T(0);
#pragma unroll
            for (uint32_t k = 0; k < count; ++k) total += part[pbase + k * outputs + v];
            Gn[gather_off<LOGD>(lam) + v] = total;
        }
        pbase += outputs < 64 ? waves << shl : uint32_t(NT);
        if (tl_count > 64) {
            const uint32_t per = tl_count >> 6;
            for (uint32_t u = tid; u < outputs; u += NT) {
                T total = T(0);
#pragma unroll
                for (uint32_t k = 0; k < per; ++k) total += part_b[pbase_b + u * per + k];
                const uint32_t q = gather_off<LOGD>(lam) + u;
                gxs[q] = (FIRST ? T(0) : gxs[q]) + c * G[q] + total;
            }
            pbase_b += outputs * per;
        }
    }
}

// R_m = c_m x + x * R_{m+1} at levels 1..n (n = N - m + 1) for m = M down to 2, a barrier after each; the word w of k
// letters takes its k - 1 cuts w = (prefix)(suffix) with compile-time shifts, so its loads do not wait for one another.
template <typename T, int LOGD, int NT, int N, int M>
__device__ __forceinline__ void gather_horner(const T *__restrict__ xs, T *__restrict__ rs, uint32_t tid)
{
    if constexpr (M >= 2) {
        constexpr int n = N - M + 1;
        const T c = (M & 1 ? T(1) : T(-1)) / T(M);
        uint32_t o_out = 0, o_next = 0;   // R_M and R_{M+1} inside rs (R_N first)
        for (int mm = N; mm > M; --mm) o_out += gather_off<LOGD>(N - mm + 2);
        for (int mm = N; mm > M + 1; --mm) o_next += gather_off<LOGD>(N - mm + 2);
        T *r_out = rs + o_out;
        const T *r_next = rs + o_next;
#pragma unroll
        for (int k = 1; k <= n; ++k) {
            constexpr uint32_t one = 1;
            const uint32_t cnt = one << uint32_t(LOGD * k);
            for (uint32_t w = tid; w < cnt; w += NT) {
                T acc = c * xs[gather_off<LOGD>(k) + w];
                if constexpr (M < N) {
#pragma unroll
                    for (int j = 1; j <= k - 1; ++j) {   // prefix of j letters, suffix of k - j
                        const uint32_t sh = uint32_t(LOGD * (k - j));
                        acc += xs[gather_off<LOGD>(j) + (w >> sh)] * r_next[gather_off<LOGD>(k - j) + (w & ((one << sh) - 1))];
                    }
                }
                r_out[gather_off<LOGD>(k) + w] = acc;
            }
        }
        __syncthreads();
        gather_horner<T, LOGD, NT, N, M - 1>(xs, rs, tid);
    }
}

// Steps m = M .. N-1 of the reverse pass, the depth of G_m a compile-time constant in each.
template <typename T, int LOGD, int NT, int N, int M>
__device__ __forceinline__ void gather_steps(T *gbuf, uint32_t s_low, const T *rs, const T *xs, T *gxs, T *part, T *part_b,
                                             uint32_t tid)
{
    if constexpr (M <= N - 1) {
        constexpr int n = N - M + 1;
        // R_{M+1} inside rs (R_N first), G_M and G_{M+1} inside the two cotangent buffers
        uint32_t r_off = 0;
        for (int mm = N; mm > M + 1; --mm) r_off += gather_off<LOGD>(N - mm + 2);
        const T c = (M & 1 ? T(1) : T(-1)) / T(M);
        gather_step<T, LOGD, NT, n, false>(c, static_cast<const T *>(gbuf + (M & 1) * s_low), gbuf + ((M + 1) & 1) * s_low,
                                           rs + r_off, xs, gxs, part, part_b, tid);
        __syncthreads();
        gather_steps<T, LOGD, NT, N, M + 1>(gbuf, s_low, rs, xs, gxs, part, part_b, tid);
    }
}

template <typename T, int LOGD, int NT, int N>
__global__ void __launch_bounds__(NT)
log_bwd_gather_kernel(int64_t rows, const T *__restrict__ x_g, const T *__restrict__ g_g, T *__restrict__ gx_g)
{
    extern __shared__ __align__(16) unsigned char lb_smem[];
    constexpr uint32_t d = 1u << LOGD;
    constexpr uint32_t S = gather_off<LOGD>(N + 1), S_low = gather_off<LOGD>(N);
    uint32_t r_stride_c = 0;
    for (int k = 1; k <= N - 1; ++k) r_stride_c += gather_off<LOGD>(k + 1);
    const uint32_t r_stride = r_stride_c;
    const uint32_t tid = threadIdx.x;
    T *xs = reinterpret_cast<T *>(lb_smem);
    T *Rs = xs + S;
    T *gbuf = Rs + r_stride;                                   // two cotangent buffers of S(N-1) scalars: G_m at (m & 1)
    T *gxs = gbuf + 2 * S_low;
    T *part = gxs + S;                                         // partial sums of one step
    T *part_b = part + gather_partials<LOGD>(N, NT);
    auto coef = [](int m) { return (m & 1 ? T(1) : T(-1)) / T(m); };
    auto r_at = [&](int m) {   // R_m inside Rs: R_N first
        uint32_t o = 0;
        for (int mm = N; mm > m; --mm) o += gather_off<LOGD>(N - mm + 2);
        return Rs + o;
    };

    for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
        const T *g_row = g_g + row * S;
        __syncthreads();   // the previous signature's gradient has been written out
        for (uint32_t i = tid; i < S; i += NT) xs[i] = x_g[row * S + i];
        __syncthreads();
        gather_horner<T, LOGD, NT, N, N>(xs, Rs, tid);
        if constexpr (N >= 2) {
            gather_step<T, LOGD, NT, N, true>(coef(1), g_row, gbuf + (2 & 1) * S_low, static_cast<const T *>(r_at(2)), xs, gxs, part,
                                              part_b, tid);
            __syncthreads();
            gather_steps<T, LOGD, NT, N, 2>(gbuf, S_low, Rs, xs, gxs, part, part_b, tid);
        }
        // G_N has one level
        const T *G_last = gbuf + (N & 1) * S_low;
        if (tid < d) gxs[tid] += coef(N) * G_last[tid];
        __syncthreads();
        for (uint32_t i = tid; i < S; i += NT) gx_g[row * S + i] = gxs[i];
    }
}

template <typename T>
__global__ void __launch_bounds__(kLbThreads)
fill_zero_kernel(T *__restrict__ p, int64_t n)
{
    for (int64_t i = int64_t(blockIdx.x) * kLbThreads + threadIdx.x; i < n; i += int64_t(gridDim.x) * kLbThreads) p[i] = T(0);
}

template <typename T>
__global__ void __launch_bounds__(kLbThreads)
scatter_kernel(const T *__restrict__ in, const int64_t *__restrict__ index, int64_t n, int64_t rows, T *__restrict__ out,
               int64_t out_stride)
{
    for (int64_t r = blockIdx.y; r < rows; r += gridDim.y)
        for (int64_t i = int64_t(blockIdx.x) * kLbThreads + threadIdx.x; i < n; i += int64_t(gridDim.x) * kLbThreads)
            out[r * out_stride + index[i]] = in[r * n + i];
}

int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }

// The work of the step whose cotangent G has n levels (n >= 2).
LbStep plan_step(const Shape &sh, int n)
{
    LbStep stp{};
    stp.count = n - 1;
    stp.S_next = uint32_t(sh.off[n]);
    stp.S_cur = uint32_t(sh.off[n + 1]);
    uint32_t wg = 0;
    int64_t a_off = 0, b_off = 0;
    for (int l = 1; l <= n - 1; ++l) {
        LbLevel &lv = stp.lv[l - 1];
        lv.C = uint32_t(sh.pw[l]);
        lv.U = uint32_t(sh.off[n - l + 1]);
        lv.base = uint32_t(sh.off[l + 1]);
        lv.wg_start = wg;
        if (lv.C <= uint32_t(kLbThreads)) {
            lv.wide = 0;
            lv.rpw = uint32_t(kLbThreads) / lv.C;
            uint32_t tpr = uint32_t(kLbThreads) / lv.rpw;
            tpr = tpr > 64 ? 64 : tpr;
            lv.lg_tpr = 0;
            while ((2u << lv.lg_tpr) <= tpr) ++lv.lg_tpr;
            const uint32_t groups = (lv.U + lv.rpw - 1) / lv.rpw;
            uint32_t passes = (groups + kLbMaxPartials - 1) / kLbMaxPartials;
            passes = passes < 4 ? 4 : passes;
            lv.rows_per_wg = passes * lv.rpw;
            lv.tiles = 1;
            lv.chunks = (lv.U + lv.rows_per_wg - 1) / lv.rows_per_wg;
            wg += lv.chunks;
        } else {
            lv.wide = 1;
            lv.rpw = 1;
            lv.lg_tpr = 0;
            lv.rows_per_wg = (lv.U + kLbMaxPartials - 1) / kLbMaxPartials;
            lv.rows_per_wg = lv.rows_per_wg < uint32_t(kLbWideRows) ? uint32_t(kLbWideRows) : lv.rows_per_wg;
            lv.rows_per_wg = lv.rows_per_wg < lv.U ? lv.rows_per_wg : lv.U;
            lv.tiles = (lv.C + kLbThreads * kLbWideCols - 1) / (kLbThreads * kLbWideCols);
            lv.chunks = (lv.U + lv.rows_per_wg - 1) / lv.rows_per_wg;
            wg += lv.tiles * lv.chunks;
        }
        lv.apart_off = a_off;
        lv.bpart_off = b_off;
        a_off += int64_t(lv.chunks) * lv.C;
        b_off += int64_t(lv.tiles) * lv.U;
    }
    stp.wgs = wg;
    stp.apart_stride = a_off;
    stp.bpart_stride = b_off;
    return stp;
}

struct LbWorkspace {
    int64_t r_stride;    // scalars of R_2..R_N per batch row
    int64_t g_stride;    // S(N - 1)
    int64_t r_off, g0_off, g1_off, a_off, b_off, total;   // in bytes
};

LbWorkspace plan_workspace(const Shape &sh, int64_t elem)
{
    LbWorkspace ws{};
    for (int n = 1; n <= sh.N - 1; ++n) ws.r_stride += sh.off[n + 1];
    ws.g_stride = sh.N >= 2 ? sh.off[sh.N] : 0;
    const LbStep first = sh.N >= 2 ? plan_step(sh, sh.N) : LbStep{};
    int64_t at = 0;
    auto take = [&](int64_t scalars) {
        const int64_t here = at;
        at += round_up(scalars * sh.B * elem, 256);
        return here;
    };
    ws.r_off = take(ws.r_stride);
    ws.g0_off = take(ws.g_stride);
    ws.g1_off = take(ws.g_stride);
    ws.a_off = take(first.apart_stride);
    ws.b_off = take(first.bpart_stride);
    ws.total = at;
    return ws;
}

// The single-launch kernel: its workgroup size, the LDS it needs (x, the R_m, two cotangent buffers, the gradient,
// products and wavefront sums) and when it is used.  Measured against the chain of launches at d = 4, L = 128:
// N <= 5 (S <= 1364): 14-34 us against 31-61 whatever the batch; N = 6 (S = 5460): 60 us against 73 at 32 signatures,
// but 186-230 us against 174 at 1024, where a compute unit holds one or two signatures at a time.
constexpr size_t kLbFusedMaxLds = 128 * 1024;
constexpr int64_t kLbFusedSmall = 2048;   // scalars up to which the kernel is used at any batch size
int fused_threads(const Shape &sh) { return sh.S <= kLbFusedSmall ? 256 : 1024; }
int gather_threads(const Shape &sh) { return sh.S <= kLbFusedSmall ? 256 : 512; }   // as instantiated in launch_gather
size_t fused_lds_bytes(const Shape &sh, const LbWorkspace &ws, size_t elem)
{
    const int nt = fused_threads(sh);
    return size_t(2 * sh.S + ws.r_stride + 2 * ws.g_stride + 2 * kFusedRows * nt + nt / 64) * elem;
}
// The gather form of the single-launch kernel: d = 2 to depth 10, d = 4 to depth 6, d = 8 to depth 4 (the depths
// instantiated below); LDS for x, the R_m, two cotangent buffers, the gradient and the partial sums.
int gather_log_d(const Shape &sh)
{
    if (sh.N < 2) return 0;
    return sh.d == 2 && sh.N <= 10 ? 1 : sh.d == 4 && sh.N <= 6 ? 2 : sh.d == 8 && sh.N <= 4 ? 3 : 0;
}
size_t gather_lds_bytes(const Shape &sh, const LbWorkspace &ws, size_t elem)
{
    const uint32_t nt = uint32_t(gather_threads(sh));
    const uint32_t partials = sh.d == 2 ? gather_partials<1>(sh.N, nt) : sh.d == 4 ? gather_partials<2>(sh.N, nt)
                                                                                    : gather_partials<3>(sh.N, nt);
    return size_t(2 * sh.S + ws.r_stride + 2 * ws.g_stride + partials + kGatherPartB) * elem;
}
bool use_gather(const Shape &sh, const LbWorkspace &ws, size_t elem)
{
    // up to what one workgroup may have on this device (160 KB) less a margin
    return gather_log_d(sh) != 0 && gather_lds_bytes(sh, ws, elem) <= 159 * 1024;
}
bool use_fused(const Shape &sh, const LbWorkspace &ws, size_t elem)
{
    if (use_gather(sh, ws, elem)) return true;
    return fused_lds_bytes(sh, ws, elem) <= kLbFusedMaxLds && (sh.S <= kLbFusedSmall || sh.B <= 256);
}

// offset, inside a batch row's share of the R buffer, of R_m (m = 2..N): R_N first
int64_t r_offset(const Shape &sh, int m)
{
    int64_t off = 0;
    for (int mm = sh.N; mm > m; --mm) off += sh.off[sh.N - mm + 2];
    return off;
}

template <typename T, int D>
void launch_horner(const Shape &sh, int n, T c_m, const T *x, const T *r_next, T *r_out, int64_t r_stride, hipStream_t st)
{
    const int64_t threads = sh.B * sh.off[n + 1];
    hipLaunchKernelGGL((log_bwd_horner_kernel<T, D>), dim3(unsigned((threads + kLbThreads - 1) / kLbThreads)), dim3(kLbThreads),
                       0, st, sh, n, c_m, x, r_next, r_out, r_stride);
}

template <typename T, int LOGD, int NT, int N>
hipError_t launch_gather_n(const Shape &sh, size_t lds, const T *x, const T *g, T *gx, hipStream_t st)
{
    auto kernel = log_bwd_gather_kernel<T, LOGD, NT, N>;
    if (lds > 64 * 1024) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, int(lds));
        if (e != hipSuccess) return e;
    }
    const unsigned grid = unsigned(sh.B < (int64_t(1) << 20) ? sh.B : (int64_t(1) << 20));
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(NT), lds, st, sh.B, x, g, gx);
    return hipGetLastError();
}

// The workgroup size follows from the size of a signature (gather_threads): 256 threads up to 2048 scalars, 512 beyond.
template <typename T>
hipError_t launch_gather(const Shape &sh, size_t lds, const T *x, const T *g, T *gx, hipStream_t st)
{
    switch (sh.d * 100 + sh.N) {
        case 202: return launch_gather_n<T, 1, 256, 2>(sh, lds, x, g, gx, st);
        case 203: return launch_gather_n<T, 1, 256, 3>(sh, lds, x, g, gx, st);
        case 204: return launch_gather_n<T, 1, 256, 4>(sh, lds, x, g, gx, st);
        case 205: return launch_gather_n<T, 1, 256, 5>(sh, lds, x, g, gx, st);
        case 206: return launch_gather_n<T, 1, 256, 6>(sh, lds, x, g, gx, st);
        case 207: return launch_gather_n<T, 1, 256, 7>(sh, lds, x, g, gx, st);
        case 208: return launch_gather_n<T, 1, 256, 8>(sh, lds, x, g, gx, st);
        case 209: return launch_gather_n<T, 1, 256, 9>(sh, lds, x, g, gx, st);
        case 210: return launch_gather_n<T, 1, 256, 10>(sh, lds, x, g, gx, st);
        case 402: return launch_gather_n<T, 2, 256, 2>(sh, lds, x, g, gx, st);
        case 403: return launch_gather_n<T, 2, 256, 3>(sh, lds, x, g, gx, st);
        case 404: return launch_gather_n<T, 2, 256, 4>(sh, lds, x, g, gx, st);
        case 405: return launch_gather_n<T, 2, 256, 5>(sh, lds, x, g, gx, st);
        case 406: return launch_gather_n<T, 2, 512, 6>(sh, lds, x, g, gx, st);
        case 802: return launch_gather_n<T, 3, 256, 2>(sh, lds, x, g, gx, st);
        case 803: return launch_gather_n<T, 3, 256, 3>(sh, lds, x, g, gx, st);
        case 804: return launch_gather_n<T, 3, 512, 4>(sh, lds, x, g, gx, st);
    }
    return hipErrorNotSupported;
}

template <typename T>
hipError_t launch_log_backward(const Shape &sh, const T *x, const T *g, T *gx, void *workspace, hipStream_t st)
{
    const int N = sh.N;
    if (N == 1) return hipMemcpyAsync(gx, g, size_t(sh.B * sh.S) * sizeof(T), hipMemcpyDeviceToDevice, st);
    const LbWorkspace ws = plan_workspace(sh, int64_t(sizeof(T)));
    if (use_gather(sh, ws, sizeof(T))) return launch_gather<T>(sh, gather_lds_bytes(sh, ws, sizeof(T)), x, g, gx, st);
    if (use_fused(sh, ws, sizeof(T))) {
        const size_t fused_lds = fused_lds_bytes(sh, ws, sizeof(T));
        const bool small = fused_threads(sh) == 256;
        auto kernel = small ? log_bwd_fused_kernel<T, 256> : log_bwd_fused_kernel<T, 1024>;
        if (fused_lds > 64 * 1024) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, int(fused_lds));
            if (e != hipSuccess) return e;
        }
        const unsigned grid = unsigned(sh.B < (int64_t(1) << 20) ? sh.B : (int64_t(1) << 20));
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(small ? 256 : 1024), fused_lds, st, sh, ws.r_stride, x, g, gx);
        return hipGetLastError();
    }
    char *base = static_cast<char *>(workspace);
    T *Rs = reinterpret_cast<T *>(base + ws.r_off);
    T *Gb[2] = {reinterpret_cast<T *>(base + ws.g0_off), reinterpret_cast<T *>(base + ws.g1_off)};
    T *apart = reinterpret_cast<T *>(base + ws.a_off);
    T *bpart = reinterpret_cast<T *>(base + ws.b_off);
    auto coef = [](int m) { return (m & 1 ? T(1) : T(-1)) / T(m); };

    for (int m = N; m >= 2; --m) {
        const int n = N - m + 1;
        const T *r_next = m == N ? nullptr : Rs + r_offset(sh, m + 1);
        T *r_out = Rs + r_offset(sh, m);
        switch (sh.d) {
            case 2: launch_horner<T, 2>(sh, n, coef(m), x, r_next, r_out, ws.r_stride, st); break;
            case 3: launch_horner<T, 3>(sh, n, coef(m), x, r_next, r_out, ws.r_stride, st); break;
            case 4: launch_horner<T, 4>(sh, n, coef(m), x, r_next, r_out, ws.r_stride, st); break;
            case 5: launch_horner<T, 5>(sh, n, coef(m), x, r_next, r_out, ws.r_stride, st); break;
            case 6: launch_horner<T, 6>(sh, n, coef(m), x, r_next, r_out, ws.r_stride, st); break;
            case 7: launch_horner<T, 7>(sh, n, coef(m), x, r_next, r_out, ws.r_stride, st); break;
            case 8: launch_horner<T, 8>(sh, n, coef(m), x, r_next, r_out, ws.r_stride, st); break;
            default: launch_horner<T, 0>(sh, n, coef(m), x, r_next, r_out, ws.r_stride, st); break;
        }
        const hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    for (int m = 1; m <= N - 1; ++m) {
        const int n = N - m + 1;
        const LbStep stp = plan_step(sh, n);
        const T *G = m == 1 ? g : Gb[m & 1];
        const int64_t g_stride = m == 1 ? sh.S : ws.g_stride;
        T *G_next = Gb[(m + 1) & 1];
        const int64_t wgs = sh.B * int64_t(stp.wgs);
        if (wgs > 0x7fffffff) return hipErrorNotSupported;
        hipLaunchKernelGGL((log_bwd_main_kernel<T>), dim3(unsigned(wgs)), dim3(kLbThreads), 0, st, stp, x, sh.S, int64_t(1), G, g_stride,
                           Rs + r_offset(sh, m + 1), ws.r_stride, apart, bpart);
        hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
        const int64_t threads = sh.B * (int64_t(stp.S_next) + stp.S_cur);
        hipLaunchKernelGGL((log_bwd_finish_kernel<T>), dim3(unsigned((threads + kLbThreads - 1) / kLbThreads)), dim3(kLbThreads),
                           0, st, stp, sh.B, coef(m), coef(N), int(m == 1), int(m == N - 1), 0, G, g_stride, apart, bpart, G_next,
                           ws.g_stride, gx, sh.S);
        err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    return hipSuccess;
}

// Gradient of out = a [x] b: grad_a[u] = g[u] + sum_v g[u v] b[v], grad_b[v] = g[v] + sum_u a[u] g[u v]: one step of the
// scheme above with x = a, R = b, G = g and unit coefficients.
// out[b][s] = sum over the rows s of group b, summed in the order of s.
template <typename T>
__global__ void __launch_bounds__(kLbThreads)
group_sum_kernel(const T *__restrict__ in, int64_t groups, int64_t group, int64_t S, T *__restrict__ out)
{
    const int64_t total = groups * S;
    for (int64_t i = int64_t(blockIdx.x) * kLbThreads + threadIdx.x; i < total; i += int64_t(gridDim.x) * kLbThreads) {
        const int64_t b = i / S, q = i - b * S;
        const T *p = in + b * group * S + q;
        T s = T(0);
        for (int64_t r = 0; r < group; ++r) s += p[r * S];
        out[i] = s;
    }
}

// The gradient of the rows a[r / a_group] [x] b[r]; with a_group > 1 the per-row gradients of the left factor go to
// the end of the workspace and are summed over each group afterwards.
template <typename T>
hipError_t launch_combine_backward(const Shape &sh, const T *a, const T *b, const T *g, T *ga, T *gb, void *workspace,
                                   hipStream_t st, int64_t a_group = 1)
{
    const LbWorkspace ws = plan_workspace(sh, int64_t(sizeof(T)));
    char *base = static_cast<char *>(workspace);
    T *ga_rows = a_group > 1 ? reinterpret_cast<T *>(base + ((ws.total + 255) / 256) * 256) : ga;
    const int64_t groups = sh.B / a_group;
    const int64_t sum_wgs = (groups * sh.S + kLbThreads - 1) / kLbThreads;
    const unsigned sum_grid = unsigned(sum_wgs < 65536 ? sum_wgs : 65536);
    if (sh.N == 1) {
        hipError_t err = hipMemcpyAsync(gb, g, size_t(sh.B * sh.S) * sizeof(T), hipMemcpyDeviceToDevice, st);
        if (err != hipSuccess) return err;
        if (a_group == 1) return hipMemcpyAsync(ga, g, size_t(sh.B * sh.S) * sizeof(T), hipMemcpyDeviceToDevice, st);
        hipLaunchKernelGGL((group_sum_kernel<T>), dim3(sum_grid), dim3(kLbThreads), 0, st, g, groups, a_group, int64_t(sh.S), ga);
        return hipGetLastError();
    }
    T *apart = reinterpret_cast<T *>(base + ws.a_off);
    T *bpart = reinterpret_cast<T *>(base + ws.b_off);
    const LbStep stp = plan_step(sh, sh.N);
    const int64_t wgs = sh.B * int64_t(stp.wgs);
    if (wgs > 0x7fffffff) return hipErrorNotSupported;
    hipLaunchKernelGGL((log_bwd_main_kernel<T>), dim3(unsigned(wgs)), dim3(kLbThreads), 0, st, stp, a, sh.S, a_group, g, sh.S, b,
                       sh.S, apart, bpart);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    const int64_t threads = sh.B * 2 * int64_t(stp.S_cur);
    hipLaunchKernelGGL((log_bwd_finish_kernel<T>), dim3(unsigned((threads + kLbThreads - 1) / kLbThreads)), dim3(kLbThreads), 0,
                       st, stp, sh.B, T(1), T(0), 1, 0, 1, g, sh.S, apart, bpart, gb, sh.S, ga_rows, sh.S);
    err = hipGetLastError();
    if (err != hipSuccess || a_group == 1) return err;
    hipLaunchKernelGGL((group_sum_kernel<T>), dim3(sum_grid), dim3(kLbThreads), 0, st, ga_rows, groups, a_group, int64_t(sh.S), ga);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_scatter(const Shape &sh, const T *in, const int64_t *index, int64_t n, T *out, hipStream_t st)
{
    const int64_t total = sh.B * sh.S;
    const int64_t fill_groups = (total + kLbThreads - 1) / kLbThreads;
    hipLaunchKernelGGL((fill_zero_kernel<T>), dim3(unsigned(fill_groups < 65536 ? fill_groups : 65536)), dim3(kLbThreads), 0, st,
                       out, total);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || n == 0) return err;
    const unsigned bx = unsigned((n + kLbThreads - 1) / kLbThreads < 4096 ? (n + kLbThreads - 1) / kLbThreads : 4096);
    const unsigned by = unsigned(sh.B < 65535 ? sh.B : 65535);
    hipLaunchKernelGGL((scatter_kernel<T>), dim3(bx, by), dim3(kLbThreads), 0, st, in, index, n, sh.B, out, sh.S);
    return hipGetLastError();
}

}  // namespace

int64_t log_backward_workspace_bytes(const Shape &sh, sig_dtype dtype)
{
    const int64_t elem = dtype == SIG_F32 ? int64_t(sizeof(float)) : int64_t(sizeof(double));
    const LbWorkspace ws = plan_workspace(sh, elem);
    return sh.N >= 2 && use_fused(sh, ws, size_t(elem)) ? 0 : ws.total;   // the single-launch kernel needs none
}

int64_t combine_backward_workspace_bytes(const Shape &sh, sig_dtype dtype)
{
    return plan_workspace(sh, dtype == SIG_F32 ? int64_t(sizeof(float)) : int64_t(sizeof(double))).total;
}

int64_t combine_grouped_backward_workspace_bytes(const Shape &sh, sig_dtype dtype)
{
    const int64_t elem = dtype == SIG_F32 ? int64_t(sizeof(float)) : int64_t(sizeof(double));
    return ((plan_workspace(sh, elem).total + 255) / 256) * 256 + sh.B * sh.S * elem;
}

hipError_t launch_log_backward_f32(const Shape &sh, const float *sig, const float *grad_log, float *grad_sig, void *workspace,
                                   hipStream_t st)
{
    return launch_log_backward<float>(sh, sig, grad_log, grad_sig, workspace, st);
}

hipError_t launch_log_backward_f64(const Shape &sh, const double *sig, const double *grad_log, double *grad_sig, void *workspace,
                                   hipStream_t st)
{
    return launch_log_backward<double>(sh, sig, grad_log, grad_sig, workspace, st);
}

hipError_t launch_combine_backward_f32(const Shape &sh, const float *a, const float *b, const float *g, float *ga, float *gb,
                                       void *workspace, hipStream_t st)
{
    return launch_combine_backward<float>(sh, a, b, g, ga, gb, workspace, st);
}

hipError_t launch_combine_backward_f64(const Shape &sh, const double *a, const double *b, const double *g, double *ga, double *gb,
                                       void *workspace, hipStream_t st)
{
    return launch_combine_backward<double>(sh, a, b, g, ga, gb, workspace, st);
}

hipError_t launch_combine_grouped_backward_f32(const Shape &sh, int64_t group, const float *a, const float *b, const float *g,
                                               float *ga, float *gb, void *workspace, hipStream_t st)
{
    return launch_combine_backward<float>(sh, a, b, g, ga, gb, workspace, st, group);
}

hipError_t launch_combine_grouped_backward_f64(const Shape &sh, int64_t group, const double *a, const double *b, const double *g,
                                               double *ga, double *gb, void *workspace, hipStream_t st)
{
    return launch_combine_backward<double>(sh, a, b, g, ga, gb, workspace, st, group);
}

hipError_t launch_scatter_f32(const Shape &sh, const float *in, const int64_t *index, int64_t n, float *out, hipStream_t st)
{
    return launch_scatter<float>(sh, in, index, n, out, st);
}

hipError_t launch_scatter_f64(const Shape &sh, const double *in, const int64_t *index, int64_t n, double *out, hipStream_t st)
{
    return launch_scatter<double>(sh, in, index, n, out, st);
}

}  // namespace sig
