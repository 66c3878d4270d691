// ReLU-gradient and bias-gradient of a [rows, k] activation matrix:
//   g = dy * [y_saved > 0]   (optionally stored),   dbias[j] = sum_rows g[., j].
// HBM-bound: every element of dy and y_saved is read once with 16-byte loads.  A block owns
// a group of 16-byte column chunks and a strided set of rows, so a thread always sees the
// same 8 columns and keeps 8 fp32 running sums in registers.  Threads of a wavefront that
// share a column chunk are combined with wavefront shuffles, wavefronts through LDS, blocks
// through a [row_blocks][k] scratch array that a second kernel sums in a fixed order.
#include "dp_kernels.h"

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

namespace {

constexpr int NT = 256;
constexpr int MAX_ROW_BLOCKS = 512;

__device__ __forceinline__ float bf16_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ unsigned keep_bits(unsigned yw)
{
    unsigned lo = (((yw & 0xffffu) - 1u) < 0x7f80u) ? 0xffffu : 0u;
    unsigned hi = (((yw >> 16) - 1u) < 0x7f80u) ? 0xffff0000u : 0u;
    return lo | hi;
}

// cgb = column chunks per block (<= 256), rpi = rows per iteration = 256 / cgb
__global__ __launch_bounds__(NT) void k_rbg_bf16(long long rows, int k, int cgb, int rpi, const unsigned short *dy,
                                                 const unsigned short *ym, unsigned short *g_out, float *ws)
{
    __shared__ float sm[NT][8];
    const int t = threadIdx.x;
    const int cl = t % cgb, rsub = t / cgb;
    const int cg = blockIdx.x * cgb + cl;
    const bool active = rsub < rpi && cg * 8 < k;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (active) {
        const long long rstep = (long long)gridDim.y * rpi;
        long long r = (long long)blockIdx.y * rpi + rsub;
        // four rows per iteration: eight independent 16-byte loads in flight per thread
        for (; r + 3 * rstep < rows; r += 4 * rstep) {
            u32x4 v[4], y[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const size_t o = (size_t)(r + u * rstep) * k + (size_t)cg * 8;
                v[u] = *reinterpret_cast<const u32x4 *>(dy + o);
                if (ym != nullptr) y[u] = *reinterpret_cast<const u32x4 *>(ym + o);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const size_t o = (size_t)(r + u * rstep) * k + (size_t)cg * 8;
                if (ym != nullptr) {
                    v[u].x &= keep_bits(y[u].x); v[u].y &= keep_bits(y[u].y); v[u].z &= keep_bits(y[u].z); v[u].w &= keep_bits(y[u].w);
                }
                if (g_out != nullptr) *reinterpret_cast<u32x4 *>(g_out + o) = v[u];
                acc[0] += bf16_lo(v[u].x); acc[1] += bf16_hi(v[u].x); acc[2] += bf16_lo(v[u].y); acc[3] += bf16_hi(v[u].y);
                acc[4] += bf16_lo(v[u].z); acc[5] += bf16_hi(v[u].z); acc[6] += bf16_lo(v[u].w); acc[7] += bf16_hi(v[u].w);
            }
        }
        for (; r < rows; r += rstep) {
            const size_t o = (size_t)r * k + (size_t)cg * 8;
            u32x4 v = *reinterpret_cast<const u32x4 *>(dy + o);
            if (ym != nullptr) {
                u32x4 y = *reinterpret_cast<const u32x4 *>(ym + o);
                v.x &= keep_bits(y.x); v.y &= keep_bits(y.y); v.z &= keep_bits(y.z); v.w &= keep_bits(y.w);
            }
            if (g_out != nullptr) *reinterpret_cast<u32x4 *>(g_out + o) = v;
            acc[0] += bf16_lo(v.x); acc[1] += bf16_hi(v.x); acc[2] += bf16_lo(v.y); acc[3] += bf16_hi(v.y);
            acc[4] += bf16_lo(v.z); acc[5] += bf16_hi(v.z); acc[6] += bf16_lo(v.w); acc[7] += bf16_hi(v.w);
        }
    }
    if (ws == nullptr) return;
    // lanes of one wavefront that hold the same column chunk: lane ids equal modulo cgb
    const bool pow2 = (cgb & (cgb - 1)) == 0;
    if (pow2 && cgb < 64) {
        for (int o = 32; o >= cgb; o >>= 1)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] += __shfl_xor(acc[i], o, 64);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) sm[t][i] = acc[i];
    __syncthreads();
    if (t < cgb && cg * 8 < k) {
        float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (pow2 && cgb < 64) {
            for (int wv = 0; wv < NT / 64; ++wv)   // lane cl of every wavefront holds that wavefront's total
#pragma unroll
                for (int i = 0; i < 8; ++i) s[i] += sm[wv * 64 + cl][i];
        } else {
            for (int u = cl; u < rpi * cgb; u += cgb)
#pragma unroll
                for (int i = 0; i < 8; ++i) s[i] += sm[u][i];
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) ws[(size_t)blockIdx.y * k + (size_t)cg * 8 + i] = s[i];
    }
}

// generic fallback: one thread per column, rows strided over blockIdx.y
template <typename T>
__device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<unsigned short>(unsigned short v) { return __uint_as_float((unsigned)v << 16); }

template <typename T>
__global__ __launch_bounds__(64) void k_rbg_cols(long long rows, int k, const T *dy, const T *ym, T *g_out, float *ws)
{
    const int col = blockIdx.x * 64 + threadIdx.x;
    if (col >= k) return;
    float acc = 0.f;
    for (long long r = blockIdx.y; r < rows; r += gridDim.y) {
        const size_t o = (size_t)r * k + col;
        T v = dy[o];
        if (ym != nullptr && !(to_f32<T>(ym[o]) > 0.f)) v = (T)0;
        if (g_out != nullptr) g_out[o] = v;
        acc += to_f32<T>(v);
    }
    if (ws != nullptr) ws[(size_t)blockIdx.y * k + col] = acc;
}

// dbias[col] = sum over row blocks of ws[b][col], in a fixed order: 8 threads per column each sum
// every 8th row block (independent loads, 4 in flight), then the 8 part sums are added in order
__global__ __launch_bounds__(256) void k_rbg_final(int k, int row_blocks, const float *ws, float *dbias)
{
    __shared__ float sm[8][32];
    const int cl = threadIdx.x & 31, part = threadIdx.x >> 5;
    const int col = blockIdx.x * 32 + cl;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    if (col < k) {
        int b = part;
        for (; b + 24 < row_blocks; b += 32) {
            s0 += ws[(size_t)b * k + col];
            s1 += ws[(size_t)(b + 8) * k + col];
            s2 += ws[(size_t)(b + 16) * k + col];
            s3 += ws[(size_t)(b + 24) * k + col];
        }
        for (; b < row_blocks; b += 8) s0 += ws[(size_t)b * k + col];
    }
    sm[part][cl] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (part == 0 && col < k) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) s += sm[i][cl];
        dbias[col] = s;
    }
}

int row_blocks_for(long long rows, int rows_per_iter, int col_blocks)
{
    // short inputs: one block per column group walks every row and writes the bias gradient itself
    if ((rows + rows_per_iter - 1) / rows_per_iter <= 48) return 1;
    long long want = 1024 / (col_blocks > 0 ? col_blocks : 1);  // about four blocks per CU in total
    long long most = (rows + rows_per_iter - 1) / rows_per_iter;
    if (want > most) want = most;
    if (want > MAX_ROW_BLOCKS) want = MAX_ROW_BLOCKS;
    if (want < 1) want = 1;
    return (int)want;
}

}  // namespace

size_t rbg_workspace_bytes(long long rows, int k)
{
    (void)rows;
    return (size_t)MAX_ROW_BLOCKS * (size_t)k * sizeof(float);
}

hipError_t rbg_launch_partial(long long rows, int k, bool bf16, const void *dy, const void *ymask, void *g_out, float *dbias,
                              float *ws, hipStream_t st, int *row_blocks)
{
    float *wsp = dbias != nullptr ? ws : nullptr;   // replaced by dbias itself when a single row block is used
    int rb;
    if (bf16 && (k % 8) == 0) {
        int chunks = k / 8;
        int cgb = chunks < NT ? chunks : NT;
        // few rows, many columns (dense layers): narrower column groups give more blocks, each of which
        // covers several rows per iteration instead of walking the rows one by one
        int want_rpi = 1;
        while (want_rpi < 32 && (long long)want_rpi * 4 < rows) want_rpi *= 2;
        if (rows <= 128 && NT / want_rpi < cgb) cgb = NT / want_rpi;
        int rpi = NT / cgb;
        int col_blocks = (chunks + cgb - 1) / cgb;
        rb = row_blocks_for(rows, rpi, col_blocks);
        if (rb == 1 && dbias != nullptr) wsp = dbias;
        hipLaunchKernelGGL(k_rbg_bf16, dim3(col_blocks, rb), dim3(NT), 0, st, rows, k, cgb, rpi,
                           (const unsigned short *)dy, (const unsigned short *)ymask, (unsigned short *)g_out, wsp);
    } else {
        int col_blocks = (k + 63) / 64;
        rb = row_blocks_for(rows, 1, col_blocks);
        if (rb == 1 && dbias != nullptr) wsp = dbias;
        if (bf16)
            hipLaunchKernelGGL(k_rbg_cols<unsigned short>, dim3(col_blocks, rb), dim3(64), 0, st, rows, k,
                               (const unsigned short *)dy, (const unsigned short *)ymask, (unsigned short *)g_out, wsp);
        else
            hipLaunchKernelGGL(k_rbg_cols<float>, dim3(col_blocks, rb), dim3(64), 0, st, rows, k, (const float *)dy,
                               (const float *)ymask, (float *)g_out, wsp);
    }
    *row_blocks = rb;
    return hipGetLastError();
}

hipError_t rbg_launch_final(int k, int row_blocks, const float *ws, float *dbias, hipStream_t st)
{
    hipLaunchKernelGGL(k_rbg_final, dim3((k + 31) / 32), dim3(256), 0, st, k, row_blocks, ws, dbias);
    return hipGetLastError();
}

hipError_t rbg_launch(long long rows, int k, bool bf16, const void *dy, const void *ymask, void *g_out, float *dbias,
                      float *ws, hipStream_t st)
{
    int rb = 1;
    hipError_t e = rbg_launch_partial(rows, k, bf16, dy, ymask, g_out, dbias, ws, st, &rb);
    if (e != hipSuccess || dbias == nullptr || rb == 1) return e;
    return rbg_launch_final(k, rb, ws, dbias, st);
}
