// Diagonal-block step of the blocked upper Cholesky factorisation M = U^T U and
// the small helper kernels of the inversion.
//
// One workgroup factors one NB x NB diagonal block held in LDS and also inverts
// the triangular factor, because both the panel solve of the factorisation and
// the bottom level of the triangular inverse need U_kk^-1.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kfac {

constexpr int NB = 128;  // panel width of the blocked factorisation (= tile size of the engine)
constexpr int DIAG_THREADS = 256;
constexpr int DIAG_MAX_ITEMS = 80;
constexpr int PREP_MAX_ITEMS = 64;

struct DiagItem {
    float *F;    // top-left of the diagonal block inside the working copy (upper triangle valid)
    float *S;    // same block of the inverse-factor storage
    int *info;   // status word of the matrix
    int n;       // block size (<= NB)
    int ldf;
    int lds;
    int pivot_base;  // index of the block's first row in the whole matrix
};

struct DiagLaunch {
    DiagItem it[DIAG_MAX_ITEMS];
};

// In:  F block = current (already updated) diagonal block, upper triangle.
// Out: F block upper triangle = U_kk with U_kk^T U_kk = block,
//      S block upper triangle = W = U_kk^-1, S block strict lower triangle = W^T.
// A pivot that is not positive (or not finite) is recorded in *info as its
// 1-based index in the whole matrix (first failure wins) and replaced by 1 so
// that the arithmetic stays finite; the caller discards the result.
__global__ __launch_bounds__(DIAG_THREADS) void diag_block_kernel(const DiagLaunch dl)
{
    __shared__ float T[NB][NB + 1];
    __shared__ float dinv[NB];   // 1 / U[j][j]

    const DiagItem &it = dl.it[blockIdx.x];
    const int n = it.n;
    const int tid = threadIdx.x;

    for (int e = tid; e < NB * NB; e += DIAG_THREADS) {
        const int r = e / NB, c = e % NB;
        float v = 0.f;
        if (r < n && c < n && r <= c) v = it.F[(size_t)r * it.ldf + c];
        T[r][c] = v;
    }
    __syncthreads();

    // Right-looking factorisation.  Row j is final once steps < j are done; it
    // is kept unscaled in T and the scale 1/U[j][j] is kept in dinv.
    const int c = tid & (NB - 1);
    const int par = tid >> 7;  // two threads per column: rows of even / odd offset
    for (int j = 0; j < n; ++j) {
        float piv = T[j][j];
        if (!(piv > 0.f) || !(piv <= 3.0e38f)) {
            if (tid == 0) atomicCAS(it.info, 0, it.pivot_base + j + 1);
            piv = 1.f;
        }
        const float ujj = sqrtf(piv);
        const float rinv = 1.0f / ujj;
        if (tid == 0) dinv[j] = rinv;
        if (c > j && c < n) {
            const float ujc = T[j][c] * rinv;
            for (int r = j + 1 + par; r <= c; r += 2) T[r][c] -= (T[j][r] * rinv) * ujc;
        }
        __syncthreads();
        if (tid == 0 && piv == 1.f && !(T[j][j] > 0.f)) T[j][j] = 1.f;
    }
    __syncthreads();

    // U[j][c] = T[j][c] * dinv[j].  Scale in place (upper triangle, diagonal included).
    for (int e = tid; e < NB * NB; e += DIAG_THREADS) {
        const int r = e / NB, cc = e % NB;
        if (r < n && cc < n && r <= cc) T[r][cc] *= dinv[r];
    }
    __syncthreads();
    for (int e = tid; e < NB * NB; e += DIAG_THREADS) {
        const int r = e / NB, cc = e % NB;
        if (r < n && cc < n && r <= cc) it.F[(size_t)r * it.ldf + cc] = T[r][cc];
    }

    // W = U^-1 by back substitution, one column per pair of lanes: for column c,
    // W[c][c] = 1/U[c][c] and, going up, W[i][c] = -(sum_{k=i+1..c} U[i][k] W[k][c]) / U[i][i].
    // The two lanes of a pair split the sum by the parity of k and combine with a
    // shuffle.  W[i][c] (i < c) is kept at T[c][i], the unused lower triangle.
    {
        const int col = tid >> 1;  // 0..127
        const int p = tid & 1;
        const bool active = col < n;
        const float wcc = active ? dinv[col] : 0.f;
        // all lanes of a wave run the same trip count (the largest column of the wave)
        const int wave_last = min(n - 1, ((tid | 63) >> 1));
        for (int i = wave_last - 1; i >= 0; --i) {
            float part = 0.f;
            if (active && i < col) {
                // k runs over i+1..col; element k == col uses wcc
                for (int k = i + 1 + p; k <= col; k += 2) {
                    const float w = (k == col) ? wcc : T[col][k];
                    part += T[i][k] * w;
                }
            }
            const float other = __shfl_xor(part, 1);
            const float tot = part + other;
            // both lanes of the pair store the same value, so each one later reads its own write
            if (active && i < col) T[col][i] = -tot * dinv[i];
        }
    }
    __syncthreads();
    for (int e = tid; e < NB * NB; e += DIAG_THREADS) {
        const int r = e / NB, cc = e % NB;
        if (r < n && cc < n) {
            float v;
            if (r == cc) v = dinv[r];
            else if (r < cc) v = T[cc][r];  // W[r][cc]
            else v = T[r][cc];              // mirror: W[cc][r]
            it.S[(size_t)r * it.lds + cc] = v;
        }
    }
}

struct PrepItem {
    const float *src;  // caller's factor
    float *dst;        // working copy
    int *info;
    int d;
    int lds_;          // ld of src
    int ldd;           // ld of dst
};

struct PrepLaunch {
    PrepItem it[PREP_MAX_ITEMS];
    float damping;
};

__global__ void invert_clear_info_kernel(const PrepLaunch pl, int count)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) *pl.it[i].info = 0;
}

// dst = src + damping * I (full copy); a non-finite source element sets info = -1.
__global__ __launch_bounds__(256) void invert_prepare_kernel(const PrepLaunch pl)
{
    const PrepItem &it = pl.it[blockIdx.y];
    const int d = it.d;
    bool bad = false;
    for (int r = blockIdx.x; r < d; r += gridDim.x) {
        for (int c = threadIdx.x; c < d; c += blockDim.x) {
            float v = it.src[(size_t)r * it.lds_ + c];
            if (!(fabsf(v) <= 3.0e38f)) bad = true;
            if (r == c) v += pl.damping;
            it.dst[(size_t)r * it.ldd + c] = v;
        }
    }
    if (bad) atomicCAS(it.info, 0, -1);
}

}  // namespace kfac
