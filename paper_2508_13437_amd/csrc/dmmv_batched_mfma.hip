// Batched residual on the matrix cores (fp32 problems whose value set D is exact in bf16).
//
// The residual of R instances sharing X is a dense contraction: acc[i][q] = sum_j X_ij * D[k_jq],
// then r[i][q] = fma(acc, s_q, -b[i][q]).  The codes D[k] are exact in bf16, and X is cut into
// up to three bf16 planes whose sum is X exactly (8 + 8 + 8 significand bits, by truncation),
// so every product the matrix cores form is exact in fp32 and only the fp32 accumulation rounds.
// The summation order differs from the sequential kernel's, so its result agrees with that
// kernel's only to the rounding of an fp32 sum, and it is used only when the caller asks for it.
//
// Layouts: Xp[plane][m][ldk] and Qt[R][ldk] in bf16, ldk = n rounded up to the K step and
// zero-filled, so both operands of C = Xp * Qt^T are read along K.
#include "dmmv_common.h"

namespace dmmv {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr int MF_BM = 128, MF_BN = 128, MF_BK = 64;   // workgroup tile; 4 wavefronts of 64 x 64
constexpr int MF_LDS_STRIDE = MF_BK + 8;              // bf16 elements per LDS row (16-byte skew)

int64_t mfma_ldk(int64_t n) { return ceil_div(n > 0 ? n : 1, MF_BK) * MF_BK; }

// ---- X (row-major fp32 copy) -> three bf16 planes; flags which of the lower planes are needed
__global__ void k_split_bf16(int64_t m, int64_t n, int64_t ldk, const float* __restrict__ Xt,
                             uint16_t* __restrict__ Xp, int32_t* flags) {
    const int64_t t = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    const bool in = t < m * ldk;
    uint32_t hi = 0, mid = 0, lo = 0;
    if (in) {
        const int64_t i = t / ldk, j = t % ldk;
        if (j < n) {
            const float x = Xt[i * n + j];
            hi = __float_as_uint(x) & 0xFFFF0000u;
            const float rem1 = x - __uint_as_float(hi);              // exact
            mid = __float_as_uint(rem1) & 0xFFFF0000u;
            const float rem2 = rem1 - __uint_as_float(mid);          // exact, <= 8 significant bits
            lo = __float_as_uint(rem2) & 0xFFFF0000u;
        }
        Xp[t] = (uint16_t)(hi >> 16);
        Xp[m * ldk + t] = (uint16_t)(mid >> 16);
        Xp[2 * m * ldk + t] = (uint16_t)(lo >> 16);
    }
    const bool need_mid = (mid << 1) != 0, need_lo = (lo << 1) != 0;     // ignore signed zeros
    const unsigned long long bm = __ballot(need_mid), bl = __ballot(need_lo);
    if ((threadIdx.x & 63) == 0 && (bm | bl)) atomicOr(&flags[FLAG_PLANES], (bm ? 2 : 0) | (bl ? 4 : 0));
}

// ---- kidx [n][R] -> Qt[R][ldk] = bf16(D[kidx]) (exact by the create-time check), K tail zero
__global__ void k_codes_bf16(int64_t n, int64_t R, int64_t ldk, const float* __restrict__ D,
                             const int32_t* __restrict__ kidx, uint16_t* __restrict__ Qt) {
    __shared__ uint16_t tile[32][33];
    const int64_t q0 = blockIdx.x * 32ll, j0 = blockIdx.y * 32ll;
    for (int dy = threadIdx.y; dy < 32; dy += blockDim.y) {
        const int64_t j = j0 + dy, q = q0 + threadIdx.x;
        uint16_t v = 0;
        if (j < n && q < R) v = (uint16_t)(__float_as_uint(D[kidx[j * R + q]]) >> 16);
        tile[dy][threadIdx.x] = v;
    }
    __syncthreads();
    for (int dy = threadIdx.y; dy < 32; dy += blockDim.y) {
        const int64_t q = q0 + dy, j = j0 + threadIdx.x;
        if (q < R && j < ldk) Qt[q * ldk + j] = tile[threadIdx.x][dy];
    }
}

// ---- C = sum over planes Xp * Qt^T on v_mfma_f32_32x32x16_bf16, fused scale and -b ---------
// Operand layout of the instruction (wave64): lane l supplies row (A) / column (B) l % 32 with
// the 8 consecutive K elements 8 * (l / 32) .. + 7; it receives column l % 32 of the 32 x 32
// result, rows 8 * (v / 4) + 4 * (l / 32) + v % 4 for its 16 values v.
__global__ __launch_bounds__(256) void k_residual_mfma(
    int64_t m, int64_t R, int64_t ldk, int32_t planes, const uint16_t* __restrict__ Xp,
    const uint16_t* __restrict__ Qt, const float* __restrict__ scale, const float* __restrict__ Bt,
    float* __restrict__ r) {
    __shared__ __align__(16) uint16_t As[MF_BM * MF_LDS_STRIDE];
    __shared__ __align__(16) uint16_t Bs[MF_BN * MF_LDS_STRIDE];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int wm = w >> 1, wn = w & 1;
    const int64_t i0 = blockIdx.y * (int64_t)MF_BM, q0 = blockIdx.x * (int64_t)MF_BN;
    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    constexpr int CHUNKS_PER_ROW = MF_BK / 8;                       // 16-byte chunks
    constexpr int CHUNKS = MF_BM * CHUNKS_PER_ROW / 256;            // per thread and operand
    for (int s = 0; s < 3; ++s) {
        if (!(planes & (1 << s))) continue;
        const uint16_t* __restrict__ Xs = Xp + (int64_t)s * m * ldk;
        for (int64_t k0 = 0; k0 < ldk; k0 += MF_BK) {
            uint4 ra[CHUNKS], rb[CHUNKS];
#pragma unroll
            for (int u = 0; u < CHUNKS; ++u) {
                const int c = threadIdx.x + 256 * u;
                const int row = c / CHUNKS_PER_ROW, kc = (c % CHUNKS_PER_ROW) * 8;
                const int64_t gi = i0 + row, gq = q0 + row;
                ra[u] = gi < m ? *reinterpret_cast<const uint4*>(Xs + gi * ldk + k0 + kc) : make_uint4(0, 0, 0, 0);
                rb[u] = gq < R ? *reinterpret_cast<const uint4*>(Qt + gq * ldk + k0 + kc) : make_uint4(0, 0, 0, 0);
            }
            __syncthreads();                                         // previous step consumed
#pragma unroll
            for (int u = 0; u < CHUNKS; ++u) {
                const int c = threadIdx.x + 256 * u;
                const int row = c / CHUNKS_PER_ROW, kc = (c % CHUNKS_PER_ROW) * 8;
                *reinterpret_cast<uint4*>(&As[row * MF_LDS_STRIDE + kc]) = ra[u];
                *reinterpret_cast<uint4*>(&Bs[row * MF_LDS_STRIDE + kc]) = rb[u];
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < MF_BK; kk += 16) {
                bf16x8 fa[2], fb[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    fa[t] = *reinterpret_cast<const bf16x8*>(&As[(wm * 64 + t * 32 + (lane & 31)) * MF_LDS_STRIDE + kk + (lane >> 5) * 8]);
                    fb[t] = *reinterpret_cast<const bf16x8*>(&Bs[(wn * 64 + t * 32 + (lane & 31)) * MF_LDS_STRIDE + kk + (lane >> 5) * 8]);
                }
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int64_t q = q0 + wn * 64 + b * 32 + (lane & 31);
        if (q >= R) continue;
        const float sc = scale[q];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t i = i0 + wm * 64 + a * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
                if (i < m) r[i * R + q] = dmmv_fma(acc[a][b][v], sc, -Bt[i * R + q]);
            }
    }
}

// ---- host dispatch ---------------------------------------------------------------------------
dmmv_status batched_mfma_build(Ctx* c) {
    const int64_t m = c->p.m, n = c->p.n;
    if (m == 0 || n == 0) return DMMV_OK;
    const int64_t tot = m * c->mfma_ldk;
    hipLaunchKernelGGL(k_split_bf16, dim3((unsigned)ceil_div(tot, 256)), dim3(256), 0, c->stream, m, n,
                       c->mfma_ldk, (const float*)c->Xt, (uint16_t*)c->Xp, c->flags);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

dmmv_status batched_mfma_residual(Ctx* c) {
    const int64_t m = c->p.m, n = c->p.n, R = c->p.R;
    if (m == 0) return DMMV_OK;
    const int64_t ldk = c->mfma_ldk;
    dim3 gq((unsigned)ceil_div(R, 32), (unsigned)ceil_div(ldk, 32));
    hipLaunchKernelGGL(k_codes_bf16, gq, dim3(32, 8), 0, c->stream, n, R, ldk, (const float*)c->D_dev,
                       (const int32_t*)c->kidx, (uint16_t*)c->Qt);
    dim3 grid((unsigned)ceil_div(R, MF_BN), (unsigned)ceil_div(m, MF_BM));
    hipLaunchKernelGGL(k_residual_mfma, grid, dim3(256), 0, c->stream, m, R, ldk, c->mfma_planes,
                       (const uint16_t*)c->Xp, (const uint16_t*)c->Qt, (const float*)c->scale_dev,
                       (const float*)c->Bt, (float*)c->r);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

}  // namespace dmmv
