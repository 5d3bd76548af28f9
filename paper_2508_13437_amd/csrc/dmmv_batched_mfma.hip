// Batched residual on the matrix cores (fp32 problems whose value set D is exact in bf16).
//
// The residual of R instances sharing X is a dense contraction: acc[i][q] = sum_j X_ij * D[k_jq],
// then r[i][q] = fma(acc, s_q, -b[i][q]).  The codes D[k] are exact in bf16, and X is cut into
// up to three bf16 planes whose sum is X exactly (8 + 8 + 8 significand bits, by truncation),
// so every product the matrix cores form is exact in fp32 and only the fp32 accumulation rounds.
// The summation order differs from the sequential kernel's, so its result agrees with that
// kernel's only to the rounding of an fp32 sum, and it is used only when the caller asks for it.
//
// Layouts: Xp[plane][m][ldk] and Qt[R][ldk] in bf16, ldk >= n rounded up to the K step and
// zero-filled, so both operands of C = Xp * Qt^T are read along K.
#include "dmmv_common.h"

namespace dmmv {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
// 16 bytes in flight between global memory and the LDS (a plain vector type: a struct such as
// uint4 lets the optimiser fuse the load and the later store into one late copy)
typedef uint32_t mf_piece __attribute__((ext_vector_type(4)));

// Workgroup tile 256 x 256 over a K step of 64: 8 wavefronts, 2 (rows) x 4 (columns), each owning
// 128 x 64 of the result as 4 x 2 instruction tiles.  A 256 x 256 tile needs 64 KB of operands
// per 8.4 Mflop (128 flop per byte), which keeps the traffic between the L2 and the compute units
// at a quarter of what the matrix cores could consume with 128 x 128 tiles.
// When that leaves compute units without a tile, the rows are cut in 128 instead (WA = 2: each
// wavefront owns 64 x 64).
constexpr int MF_BN = 256, MF_BK = 64, MF_THREADS = 512;
constexpr int MF_LDS_STRIDE = MF_BK + 8;              // bf16 elements per LDS row (16-byte skew)
constexpr int mf_bm(int WA) { return 2 * 32 * WA; }   // rows of the workgroup tile
constexpr int mf_stage(int WA) { return (mf_bm(WA) + MF_BN) * MF_LDS_STRIDE; }   // bf16 elements per LDS stage
constexpr int mf_lds_bytes(int WA) { return 2 * mf_stage(WA) * (int)sizeof(uint16_t); }   // two stages

// Row stride of both operands: n rounded up to the K step, then to an odd number of K steps.
// A stride that is a multiple of a few KB (n = 4096 gives 8 KB) puts the same K slice of every
// row on the same L2 channel, and all workgroups of an XCD read the same K slice at the same
// time; an odd multiple of 128 bytes spreads consecutive rows over the channels.
int64_t mfma_ldk(int64_t n) { return (ceil_div(n > 0 ? n : 1, MF_BK) | 1) * MF_BK; }
static int64_t mfma_ksteps(int64_t n) { return ceil_div(n > 0 ? n : 1, MF_BK); }

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
//
// The K loop runs over (plane, K step) pairs.  The operands of step t + 1 are requested into
// registers before the matrix cores start on step t and are written to the other LDS stage after
// it, so one barrier per step suffices.  Rows past m and columns past R are clamped on the load
// (their results are never stored); the K tail is zero in both operands.
template <int WA>
__global__ __launch_bounds__(MF_THREADS) void k_residual_mfma(
    int64_t m, int64_t R, int64_t ldk, int32_t ksteps, int32_t planes, int32_t tiles_q,
    const uint16_t* __restrict__ Xp, const uint16_t* __restrict__ Qt,
    const float* __restrict__ scale, const float* __restrict__ Bt, float* __restrict__ r) {
    extern __shared__ __align__(16) uint16_t mf_lds[];
    constexpr int MF_BM = mf_bm(WA), MF_STAGE = mf_stage(WA);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;
    const int wm = w >> 2, wn = w & 3;

    // consecutive workgroups take consecutive column tiles of one row tile.  (They land on
    // different XCDs; an order that gave each XCD a compact block of tiles measured slower: more
    // workgroups then ask one L2 for the same lines at the same moment.)
    const int64_t i0 = (blockIdx.x / tiles_q) * (int64_t)MF_BM, q0 = (blockIdx.x % tiles_q) * (int64_t)MF_BN;

    floatx16 acc[WA][2];
#pragma unroll
    for (int a = 0; a < WA; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    // this thread's 16-byte chunks of a stage: rows tid / 8 + 64 u, K offset 8 (tid % 8)
    constexpr int CHA = MF_BM * (MF_BK / 8) / MF_THREADS, CHB = MF_BN * (MF_BK / 8) / MF_THREADS;
    const int crow = tid >> 3, ckc = (tid & 7) * 8;
    int64_t offA[CHA], offB[CHB];
#pragma unroll
    for (int u = 0; u < CHA; ++u) offA[u] = min(i0 + crow + 64 * u, m - 1) * ldk + ckc;
#pragma unroll
    for (int u = 0; u < CHB; ++u) offB[u] = min(q0 + crow + 64 * u, R - 1) * ldk + ckc;
    // the planes in use, ascending (plane 0 always is)
    const int n_planes = 1 + ((planes >> 1) & 1) + ((planes >> 2) & 1);
    const int plane0 = 0, plane1 = (planes & 2) ? 1 : 2, plane2 = 2;
    const int T = n_planes * ksteps;

    mf_piece ra[CHA], rb[CHB];
// (written as macros: the arrays stay in registers only if nothing takes their address)
#define MF_REQUEST(t)                                                                         \
    {                                                                                         \
        const int ps_ = (t) / ksteps;                                                         \
        const int s_ = ps_ == 0 ? plane0 : ps_ == 1 ? plane1 : plane2;                        \
        const int64_t k0_ = (int64_t)((t) % ksteps) * MF_BK;                                  \
        const uint16_t* __restrict__ Xs_ = Xp + (int64_t)s_ * m * ldk + k0_;                  \
        const uint16_t* __restrict__ Qs_ = Qt + k0_;                                          \
        _Pragma("unroll") for (int u = 0; u < CHA; ++u)                                       \
            ra[u] = *reinterpret_cast<const mf_piece*>(Xs_ + offA[u]);                        \
        _Pragma("unroll") for (int u = 0; u < CHB; ++u)                                       \
            rb[u] = *reinterpret_cast<const mf_piece*>(Qs_ + offB[u]);                        \
    }
#define MF_DEPOSIT(stage)                                                                     \
    {                                                                                         \
        uint16_t* As_ = mf_lds + (stage) * MF_STAGE;                                          \
        uint16_t* Bs_ = As_ + MF_BM * MF_LDS_STRIDE;                                          \
        _Pragma("unroll") for (int u = 0; u < CHA; ++u)                                       \
            *reinterpret_cast<mf_piece*>(&As_[(crow + 64 * u) * MF_LDS_STRIDE + ckc]) = ra[u]; \
        _Pragma("unroll") for (int u = 0; u < CHB; ++u)                                       \
            *reinterpret_cast<mf_piece*>(&Bs_[(crow + 64 * u) * MF_LDS_STRIDE + ckc]) = rb[u]; \
    }

    MF_REQUEST(0);
    MF_DEPOSIT(0);
    __syncthreads();
    const int frag = (lane & 31) * MF_LDS_STRIDE + (lane >> 5) * 8;
    for (int t = 0; t < T; ++t) {
        MF_REQUEST(min(t + 1, T - 1));          // unconditional: the last step re-reads its own operands
        asm volatile("" ::: "memory");          // keep the requests ahead of the matrix-core work:
        __builtin_amdgcn_sched_barrier(0);      // neither the optimiser nor the scheduler may sink them
        const uint16_t* As = mf_lds + (t & 1) * MF_STAGE + wm * (32 * WA) * MF_LDS_STRIDE + frag;
        const uint16_t* Bs = mf_lds + (t & 1) * MF_STAGE + (MF_BM + wn * 64) * MF_LDS_STRIDE + frag;
        bf16x8 fa[2][WA], fb[2][2];              // fragments of K slice kk and of the next one
#pragma unroll
        for (int a = 0; a < WA; ++a) fa[0][a] = *reinterpret_cast<const bf16x8*>(As + a * 32 * MF_LDS_STRIDE);
#pragma unroll
        for (int b = 0; b < 2; ++b) fb[0][b] = *reinterpret_cast<const bf16x8*>(Bs + b * 32 * MF_LDS_STRIDE);
#pragma unroll
        for (int ks = 0; ks < MF_BK / 16; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            if (ks + 1 < MF_BK / 16) {
#pragma unroll
                for (int a = 0; a < WA; ++a)
                    fa[nxt][a] = *reinterpret_cast<const bf16x8*>(As + a * 32 * MF_LDS_STRIDE + (ks + 1) * 16);
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    fb[nxt][b] = *reinterpret_cast<const bf16x8*>(Bs + b * 32 * MF_LDS_STRIDE + (ks + 1) * 16);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int a = 0; a < WA; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][a], fb[cur][b], acc[a][b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        MF_DEPOSIT((t + 1) & 1);                // after the last step nobody reads this stage
        __syncthreads();
    }
#undef MF_REQUEST
#undef MF_DEPOSIT
    // r = fma(acc, s_q, -b): the 16 values of one instruction tile are requested together (rows
    // past m clamped), so the loads overlap instead of forming one round trip per element
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int64_t q = q0 + wn * 64 + b * 32 + (lane & 31);
        if (q >= R) continue;
        const float sc = scale[q];
#pragma unroll
        for (int a = 0; a < WA; ++a) {
            const int64_t ibase = i0 + wm * (32 * WA) + a * 32 + (lane >> 5) * 4;
            float bv[16];
#pragma unroll
            for (int v = 0; v < 16; ++v)
                bv[v] = Bt[min(ibase + (v >> 2) * 8 + (v & 3), m - 1) * R + q];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t i = ibase + (v >> 2) * 8 + (v & 3);
                if (i < m) r[i * R + q] = dmmv_fma(acc[a][b][v], sc, -bv[v]);
            }
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
    const int64_t tiles_q = ceil_div(R, MF_BN);
    int dev = 0, cus = 0;
    DMMV_HIP_CHECK(hipGetDevice(&dev));
    DMMV_HIP_CHECK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const bool tall = ceil_div(m, mf_bm(4)) * tiles_q >= cus;       // 256-row tiles fill the chip
    const int64_t tiles_i = ceil_div(m, tall ? mf_bm(4) : mf_bm(2));
    if (tiles_i * tiles_q > (int64_t)1 << 30) return DMMV_ERR_UNSUPPORTED;
    const void* kern = tall ? (const void*)k_residual_mfma<4> : (const void*)k_residual_mfma<2>;
    const int lds = tall ? mf_lds_bytes(4) : mf_lds_bytes(2);
    DMMV_TRY(ensure_dynamic_lds(kern, lds));
    const unsigned grid = (unsigned)(tiles_i * tiles_q);
    hipLaunchKernelGGL(tall ? k_residual_mfma<4> : k_residual_mfma<2>, dim3(grid), dim3(MF_THREADS), lds,
                       c->stream, m, R, ldk, (int32_t)mfma_ksteps(n), c->mfma_planes, (int32_t)tiles_q,
                       (const uint16_t*)c->Xp, (const uint16_t*)c->Qt, (const float*)c->scale_dev,
                       (const float*)c->Bt, (float*)c->r);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

}  // namespace dmmv
