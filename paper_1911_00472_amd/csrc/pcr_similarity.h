// Multi-scale structural similarity of two batches of decoded pictures (the fidelity estimate of the paper's
// Section 6.4: how close the picture of scan group k is to the full one), on the device.
//
// The measure is the published one (Wang, Simoncelli and Bovik 2003): on luma, an 11 x 11 Gaussian window of
// sigma 1.5 at every position where it fits, C1 = (0.01*255)^2, C2 = (0.03*255)^2; the contrast-structure term
// averaged at scales 1 .. M-1 and luminance x contrast-structure at scale M, combined as a product of powers
// with the published exponents; each further scale is the 2 x 2 average of the one before.  M = 5, or as many
// scales as keep the smaller side at least 11 samples (with fewer than five, the exponents used are rescaled to
// sum to 1); a negative scale mean counts as 0.
//
// Layout of the work: one workgroup per 32 x 32 tile of window positions of one scale of one picture.  A
// sample of scale j is the mean of an aligned 2^j x 2^j block of the picture (what j rounds of 2 x 2 averaging
// give), taken straight from the uint8 pixels with exact integer sums, so no pyramid is ever stored.  The
// window is separable: 11 taps along rows into LDS, 11 taps down columns out of it.  Samples are centred on
// 128 before squaring, which keeps the fp32 variances (a difference of two large numbers) accurate.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pcr {

constexpr int kSsimScales = 5, kSsimWin = 11, kSsimTile = 32, kSsimIn = kSsimTile + kSsimWin - 1;     // 42

__host__ __device__ inline int ssim_scale_count(uint32_t W, uint32_t H) {
    const uint32_t m = W < H ? W : H;
    if (m < (uint32_t)kSsimWin) return 0;
    int M = 1;
    while (M < kSsimScales && (m >> M) >= (uint32_t)kSsimWin) M++;
    return M;
}
// Tiles of scale j of a W x H picture (j below its scale count), and how many lie side by side.
__host__ __device__ inline uint32_t ssim_tiles(uint32_t W, uint32_t H, int j, uint32_t* across) {
    const uint32_t ow = (W >> j) - (kSsimWin - 1), oh = (H >> j) - (kSsimWin - 1);
    *across = (ow + kSsimTile - 1) / kSsimTile;
    return *across * ((oh + kSsimTile - 1) / kSsimTile);
}
__host__ __device__ inline uint32_t ssim_tiles_all(uint32_t W, uint32_t H) {
    uint32_t t = 0, across;
    for (int j = 0, M = ssim_scale_count(W, H); j < M; j++) t += ssim_tiles(W, H, j, &across);
    return t;
}

// part[i * tiles_max + t] = (sum of contrast-structure, sum of luminance x contrast-structure) over the
// window positions of tile t of picture i; tiles are numbered scale by scale.
__global__ void __launch_bounds__(256) k_ssim_tiles(const uint32_t* __restrict__ dims, const uint64_t* __restrict__ out_off, int C,
                                                    const uint8_t* __restrict__ pa, const uint8_t* __restrict__ pb,
                                                    float2* __restrict__ part, uint32_t tiles_max) {
    __shared__ float sa[kSsimIn][kSsimIn + 1], sb[kSsimIn][kSsimIn + 1];
    __shared__ float hp[5][kSsimIn][kSsimTile + 1];
    __shared__ float g[kSsimWin];
    __shared__ float red[4][2];
    const uint32_t i = blockIdx.y, tid = threadIdx.x;
    const uint32_t W = dims[2 * i], H = dims[2 * i + 1];
    const int M = ssim_scale_count(W, H);
    uint32_t t = blockIdx.x, across = 1;
    int j = 0;
    for (; j < M; j++) {
        const uint32_t cnt = ssim_tiles(W, H, j, &across);
        if (t < cnt) break;
        t -= cnt;
    }
    if (j >= M) return;                                              // (uniform over the workgroup)
    const uint32_t Wj = W >> j, Hj = H >> j, ow = Wj - (kSsimWin - 1), oh = Hj - (kSsimWin - 1);
    const uint32_t ox = (t % across) * kSsimTile, oy = (t / across) * kSsimTile;
    if (tid < (uint32_t)kSsimWin) {
        float sum = 0;
        for (int k = 0; k < kSsimWin; k++) sum += expf(-(float)((k - 5) * (k - 5)) / 4.5f);
        g[tid] = expf(-(float)(((int)tid - 5) * ((int)tid - 5)) / 4.5f) / sum;
    }
    // samples of this scale under the tile: means of 2^j x 2^j blocks, centred on 128
    const uint32_t s = 1u << j;
    const float inv_area = 1.0f / (float)(s * s);
    const uint8_t* A = pa + out_off[i];
    const uint8_t* B = pb + out_off[i];
    for (uint32_t idx = tid; idx < (uint32_t)(kSsimIn * kSsimIn); idx += 256) {
        const uint32_t sy = idx / kSsimIn, sx = idx % kSsimIn, X = ox + sx, Y = oy + sy;
        float va = 0, vb = 0;
        if (X < Wj && Y < Hj) {
            uint32_t a0 = 0, a1 = 0, a2 = 0, b0 = 0, b1 = 0, b2 = 0;
            for (uint32_t dy = 0; dy < s; dy++) {
                const size_t row = ((size_t)(Y * s + dy) * W + (size_t)X * s) * (size_t)C;
                if (C == 3) {
                    for (uint32_t dx = 0; dx < 3 * s; dx += 3) {
                        a0 += A[row + dx]; a1 += A[row + dx + 1]; a2 += A[row + dx + 2];
                        b0 += B[row + dx]; b1 += B[row + dx + 1]; b2 += B[row + dx + 2];
                    }
                } else {
                    for (uint32_t dx = 0; dx < s; dx++) { a0 += A[row + dx]; b0 += B[row + dx]; }
                }
            }
            if (C == 3) {
                va = (0.299f * (float)a0 + 0.587f * (float)a1 + 0.114f * (float)a2) * inv_area - 128.0f;
                vb = (0.299f * (float)b0 + 0.587f * (float)b1 + 0.114f * (float)b2) * inv_area - 128.0f;
            } else {
                va = (float)a0 * inv_area - 128.0f;
                vb = (float)b0 * inv_area - 128.0f;
            }
        }
        sa[sy][sx] = va; sb[sy][sx] = vb;
    }
    __syncthreads();
    // 11 taps along the rows: weighted sums of a, b, a*a, b*b, a*b
    for (uint32_t idx = tid; idx < (uint32_t)(kSsimIn * kSsimTile); idx += 256) {
        const uint32_t y = idx / kSsimTile, x = idx % kSsimTile;
        float ma = 0, mb = 0, aa = 0, bb = 0, ab = 0;
#pragma unroll
        for (int k = 0; k < kSsimWin; k++) {
            const float w = g[k], va = sa[y][x + k], vb = sb[y][x + k];
            ma += w * va; mb += w * vb; aa += w * va * va; bb += w * vb * vb; ab += w * va * vb;
        }
        hp[0][y][x] = ma; hp[1][y][x] = mb; hp[2][y][x] = aa; hp[3][y][x] = bb; hp[4][y][x] = ab;
    }
    __syncthreads();
    // 11 taps down the columns, then the two terms at every window position inside the picture
    const float C1 = 6.5025f, C2 = 58.5225f;
    float sum_cs = 0, sum_lcs = 0;
    for (uint32_t idx = tid; idx < (uint32_t)(kSsimTile * kSsimTile); idx += 256) {
        const uint32_t y = idx / kSsimTile, x = idx % kSsimTile;
        if (ox + x >= ow || oy + y >= oh) continue;
        float ma = 0, mb = 0, aa = 0, bb = 0, ab = 0;
#pragma unroll
        for (int k = 0; k < kSsimWin; k++) {
            const float w = g[k];
            ma += w * hp[0][y + k][x]; mb += w * hp[1][y + k][x];
            aa += w * hp[2][y + k][x]; bb += w * hp[3][y + k][x]; ab += w * hp[4][y + k][x];
        }
        const float var_a = aa - ma * ma, var_b = bb - mb * mb, cov = ab - ma * mb;
        const float mua = ma + 128.0f, mub = mb + 128.0f;
        const float lum = (2.0f * mua * mub + C1) / (mua * mua + mub * mub + C1);
        const float cs = (2.0f * cov + C2) / (var_a + var_b + C2);
        sum_cs += cs; sum_lcs += lum * cs;
    }
    for (int d = 32; d > 0; d >>= 1) { sum_cs += __shfl_down(sum_cs, d); sum_lcs += __shfl_down(sum_lcs, d); }
    if ((tid & 63) == 0) { red[tid >> 6][0] = sum_cs; red[tid >> 6][1] = sum_lcs; }
    __syncthreads();
    if (tid == 0)
        part[(size_t)i * tiles_max + blockIdx.x] = make_float2(red[0][0] + red[1][0] + red[2][0] + red[3][0],
                                                               red[0][1] + red[1][1] + red[2][1] + red[3][1]);
}

// One wavefront per picture: the scale means from the tile sums (in double, in a fixed order), then the
// product of powers.  A picture too small for the window scores NaN.
__global__ void __launch_bounds__(64) k_ssim_score(const uint32_t* __restrict__ dims, const float2* __restrict__ part, uint32_t tiles_max,
                                                   float* __restrict__ scores) {
    const double weight[kSsimScales] = {0.0448, 0.2856, 0.3001, 0.2363, 0.1333};
    const uint32_t i = blockIdx.x, lane = threadIdx.x;
    const uint32_t W = dims[2 * i], H = dims[2 * i + 1];
    const int M = ssim_scale_count(W, H);
    if (M == 0) { if (lane == 0) scores[i] = __builtin_nanf(""); return; }
    double wsum = 0;
    for (int j = 0; j < M; j++) wsum += weight[j];
    if (M == kSsimScales) wsum = 1.0;                       // all five scales: the exponents as published (they sum to 1.0001)
    double score = 1.0;
    uint32_t first = 0;
    for (int j = 0; j < M; j++) {
        uint32_t across;
        const uint32_t cnt = ssim_tiles(W, H, j, &across);
        double cs = 0, lcs = 0;
        for (uint32_t t = lane; t < cnt; t += 64) {
            const float2 p = part[(size_t)i * tiles_max + first + t];
            cs += (double)p.x; lcs += (double)p.y;
        }
        for (int d = 32; d > 0; d >>= 1) { cs += __shfl_down(cs, d); lcs += __shfl_down(lcs, d); }
        const double positions = (double)((W >> j) - (kSsimWin - 1)) * (double)((H >> j) - (kSsimWin - 1));
        double term = (j == M - 1 ? lcs : cs) / positions;
        if (!(term > 0.0)) term = 0.0;
        score *= pow(term, weight[j] / wsum);
        first += cnt;
    }
    if (lane == 0) scores[i] = (float)score;
}

}  // namespace pcr
