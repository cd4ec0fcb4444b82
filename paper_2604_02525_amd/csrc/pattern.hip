// Outlier-pattern detection of one tensor (paper Sec. 4.1, App. A) and the pattern-pair -> strategy
// table (Sec. 4.2).
//
// For an operand in its logical [outer, K] shape: the variance of every outer index (over its K
// elements) and of every K index (over the outer elements); the coefficient of variation of each of
// the two variance vectors, CV = std(v) / (mean(v) + eps); each CV divided by its value for IID
// data, sqrt(2 / (samples - 1)); and the class: "outer-wise" if CV^_outer / CV^_k > tau, "K-wise" if
// CV^_k / CV^_outer > tau, else none.  In the paper's notation (A is m x k, B is k x n) outer-wise is
// Row-wise for A and Column-wise for B, K-wise is Column-wise for A and Row-wise for B.
//
// All sums are kept in fp64 (the inputs are bf16, so x and x^2 are exact in fp64 and the variances
// follow from sum and sum of squares without cancellation trouble); variances are population
// variances, as are the standard deviations of the variance vectors.
//
//   k_pattern_partial  one pass over the stored matrix S[R][C]: a workgroup takes 256 rows x 512
//                      columns and writes, per row, its sum / sum of squares over the 512 columns,
//                      and per column over the 256 rows (no atomics);
//   k_pattern_fold     adds the partials of every row and every column in a fixed order (one thread each);
//   k_pattern_finish   one workgroup forms both variance vectors and their statistics and writes the class and
//                      the four CV figures.
#include "common.h"

namespace adahop {

namespace {

constexpr int PT_ROWS = 256, PT_COLS = 512;

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_down(v, d);
    return v; // valid in lane 0
}

// rowpart[cb][r] = (sum, sumsq) of row r over column block cb; colpart[rb][c] likewise.
__global__ __launch_bounds__(256) void k_pattern_partial(const uint16_t *__restrict__ S, int64_t ld, int64_t R, int64_t C,
                                                         double2 *__restrict__ rowpart, double2 *__restrict__ colpart)
{
    __shared__ double2 scol[4][PT_COLS];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int64_t r0 = (int64_t)blockIdx.y * PT_ROWS, c0 = (int64_t)blockIdx.x * PT_COLS + lane * 8;
    const bool cok = c0 < C; // C % 8 == 0 is not required: the tail chunk is handled element-wise
    double cs[8], cq[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) cs[j] = cq[j] = 0.0;
    const bool whole = c0 + 8 <= C;
    for (int i0 = 0; i0 < PT_ROWS / 4; i0 += 8) { // eight rows of the wave at a time: their loads are in flight together
        uint4 u[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int64_t r = r0 + w + 4 * (i0 + t);
            u[t] = (r < R && whole) ? load_once16(S + r * ld + c0) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int64_t r = r0 + w + 4 * (i0 + t);
            double rs = 0.0, rq = 0.0;
            if (r < R && cok) {
                float e[8];
                if (whole) {
                    e[0] = bf16_lo(u[t].x); e[1] = bf16_hi(u[t].x); e[2] = bf16_lo(u[t].y); e[3] = bf16_hi(u[t].y);
                    e[4] = bf16_lo(u[t].z); e[5] = bf16_hi(u[t].z); e[6] = bf16_lo(u[t].w); e[7] = bf16_hi(u[t].w);
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j) e[j] = c0 + j < C ? bf16_one(S[r * ld + c0 + j]) : 0.0f;
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const double x = (double)e[j], x2 = x * x;
                    rs += x;
                    rq += x2;
                    cs[j] += x;
                    cq[j] += x2;
                }
            }
            rs = wave_sum(rs);
            rq = wave_sum(rq);
            if (lane == 0 && r < R) rowpart[(int64_t)blockIdx.x * R + r] = make_double2(rs, rq);
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) scol[w][lane * 8 + j] = make_double2(cs[j], cq[j]);
    __syncthreads();
    for (int c = tid; c < PT_COLS; c += 256) {
        const int64_t cg = (int64_t)blockIdx.x * PT_COLS + c;
        if (cg < C) {
            double2 a = scol[0][c];
            for (int v = 1; v < 4; ++v) {
                a.x += scol[v][c].x;
                a.y += scol[v][c].y;
            }
            colpart[(int64_t)blockIdx.y * C + cg] = a;
        }
    }
}

// part[i] <- sum over p of part[p * n + i], p ascending, for the rows (i < R, row_parts partials) and the columns.
// One thread per index, over the whole chip: left to the one workgroup of k_pattern_finish this sum was most of
// the detector's time (112 partials x 8192 columns x 16 bytes through one compute unit).
__global__ __launch_bounds__(256) void k_pattern_fold(double2 *__restrict__ rowpart, int row_parts, double2 *__restrict__ colpart,
                                                      int col_parts, int64_t R, int64_t C)
{
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    double2 *part = g < R ? rowpart : colpart;
    const int64_t n = g < R ? R : C, i = g < R ? g : g - R;
    const int parts = g < R ? row_parts : col_parts;
    if (i >= n) return;
    double s = 0.0, q = 0.0;
    for (int p = 0; p < parts; ++p) {
        const double2 v = part[(int64_t)p * n + i];
        s += v.x;
        q += v.y;
    }
    part[i] = make_double2(s, q);
}

// Statistics of the variance vector of one axis: n entries, entry i = sum over `parts` partials of
// part[p * n + i], each variance taken over `samples` elements.  Returns (mean, mean of squares) of
// the variances through sh (block reduction, fixed order).
__device__ void variance_stats(const double2 *__restrict__ part, int parts, int64_t n, int64_t samples, double *sh,
                               double &mean_v, double &mean_v2)
{
    double a = 0.0, b = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += blockDim.x) {
        double s = 0.0, q = 0.0;
        for (int p = 0; p < parts; ++p) {
            const double2 v = part[(int64_t)p * n + i];
            s += v.x;
            q += v.y;
        }
        const double m = s / (double)samples;
        double var = q / (double)samples - m * m;
        if (var < 0.0) var = 0.0;
        a += var;
        b += var * var;
    }
    a = wave_sum(a);
    b = wave_sum(b);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if (lane == 0) {
        sh[2 * w] = a;
        sh[2 * w + 1] = b;
    }
    __syncthreads();
    double ta = 0.0, tb = 0.0;
    for (int v = 0; v < nw; ++v) {
        ta += sh[2 * v];
        tb += sh[2 * v + 1];
    }
    mean_v = ta / (double)n;
    mean_v2 = tb / (double)n;
}

__device__ __forceinline__ double ratio_or_inf(double a, double b)
{
    if (b > 0.0) return a / b;
    return a > 0.0 ? __longlong_as_double(0x7ff0000000000000LL) : 0.0;
}

// stats_out: CV_outer, CV_k, CV^_outer, CV^_k.  rows_are_outer: the stored rows are the outer indices.
__global__ __launch_bounds__(1024) void k_pattern_finish(const double2 *__restrict__ rowpart, int row_parts,
                                                         const double2 *__restrict__ colpart, int col_parts, int64_t R,
                                                         int64_t C, int rows_are_outer, double tau, double eps,
                                                         int32_t *__restrict__ pattern_out, double *__restrict__ stats_out)
{
    __shared__ double sh[32];
    double mr, mr2, mc, mc2;
    variance_stats(rowpart, row_parts, R, C, sh, mr, mr2); // row variances: over the C columns
    variance_stats(colpart, col_parts, C, R, sh, mc, mc2); // column variances: over the R rows
    if (threadIdx.x == 0) {
        double sr = mr2 - mr * mr, sc = mc2 - mc * mc;
        sr = sr > 0.0 ? sqrt(sr) : 0.0;
        sc = sc > 0.0 ? sqrt(sc) : 0.0;
        const double cv_row = sr / (mr + eps), cv_col = sc / (mc + eps);
        const double hat_row = cv_row / sqrt(2.0 / (double)(C - 1)), hat_col = cv_col / sqrt(2.0 / (double)(R - 1));
        const double cv_outer = rows_are_outer ? cv_row : cv_col, cv_k = rows_are_outer ? cv_col : cv_row;
        const double hat_outer = rows_are_outer ? hat_row : hat_col, hat_k = rows_are_outer ? hat_col : hat_row;
        int p = ADAHOP_PATTERN_NONE;
        if (ratio_or_inf(hat_outer, hat_k) > tau)
            p = ADAHOP_PATTERN_OUTER;
        else if (ratio_or_inf(hat_k, hat_outer) > tau)
            p = ADAHOP_PATTERN_K;
        *pattern_out = p;
        stats_out[0] = cv_outer;
        stats_out[1] = cv_k;
        stats_out[2] = hat_outer;
        stats_out[3] = hat_k;
    }
}

} // namespace

static void pattern_geometry(const adahop_operand_t &x, int64_t &R, int64_t &C, int64_t &rb, int64_t &cb)
{
    R = x.k_contig ? x.outer : x.K;
    C = x.k_contig ? x.K : x.outer;
    rb = ceil_div(R, PT_ROWS);
    cb = ceil_div(C, PT_COLS);
}

size_t pattern_workspace_bytes(const adahop_operand_t &x)
{
    int64_t R, C, rb, cb;
    pattern_geometry(x, R, C, rb, cb);
    return align_up((size_t)cb * R * sizeof(double2), 256) + align_up((size_t)rb * C * sizeof(double2), 256);
}

int launch_detect_pattern(const adahop_operand_t &x, double tau, double eps, int32_t *pattern_out, double *stats_out,
                          void *workspace, hipStream_t st)
{
    int64_t R, C, rb, cb;
    pattern_geometry(x, R, C, rb, cb);
    double2 *rowpart = static_cast<double2 *>(workspace);
    double2 *colpart = reinterpret_cast<double2 *>(static_cast<char *>(workspace) + align_up((size_t)cb * R * sizeof(double2), 256));
    hipLaunchKernelGGL(k_pattern_partial, dim3((unsigned)cb, (unsigned)rb), dim3(256), 0, st,
                       static_cast<const uint16_t *>(x.data), x.ld, R, C, rowpart, colpart);
    int rc = check_launch();
    if (rc != ADAHOP_OK) return rc;
    hipLaunchKernelGGL(k_pattern_fold, dim3((unsigned)ceil_div(R + C, 256)), dim3(256), 0, st, rowpart, (int)cb, colpart, (int)rb,
                       R, C);
    rc = check_launch();
    if (rc != ADAHOP_OK) return rc;
    hipLaunchKernelGGL(k_pattern_finish, dim3(1), dim3(1024), 0, st, rowpart, 1, colpart, 1, R, C, x.k_contig ? 1 : 0, tau, eps,
                       pattern_out, stats_out);
    return check_launch();
}

} // namespace adahop
