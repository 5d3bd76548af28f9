// Batched evaluation with the fused multiply-adds on the matrix cores (fp32, nd <= 32).
//
// score[q][j][k] = max_i | fma(delta_qjk, X_ij, r_iq) |  is not a contraction (the rows are
// combined by a maximum, not a sum), but the multiply-adds themselves are an outer product with
// an added matrix: v_mfma_f32_32x32x1_2b_f32 computes D = a b^T + C on two 32 x 32 blocks with
// K = 1, i.e. exactly one fused multiply-add per element, rounded once like v_fma_f32 (checked
// bit for bit on the device, cancellation and subnormal results included).  With
//     a = 64 rows of one column of X,   b = the steps delta of 32 (instance, value) pairs for
//     that column,   C = the residuals of those instances on those rows (the same for every
//     column, so it stays in registers),
// one instruction yields 2048 pairs at twice the rate of the vector unit, which is left with the
// running maximum alone (one v_max3_f32 per two pairs).
//
// Measured on MI355X: the instruction alone issues every 66-75 cycles per SIMD (2048 multiply-adds),
// but a wavefront's v_max3_f32 chain over the PREVIOUS result (other registers) does not run
// beside it: product plus chain take 156-190 cycles per SIMD, more than the two alone (the matrix
// unit reads and writes the same vector register file).  The kernel therefore scores cfg-4-sized
// batches in 21.6 ms against 18.3 ms of the vector-unit kernel, which stays the default; this one
// is selected with options.batched_eval = 2 and gives the same bits.
//
// Layout of the instruction (wave64): lane l supplies a[32 * (l / 32) + l % 32] and
// b[l % 32]; it receives, in register v, block v / 16, column l % 32 and row
// 8 * ((v % 16) / 4) + 4 * (l / 32) + v % 4 of that block.  So a lane owns one (instance, value)
// pair and sees 32 of the 64 rows: the maximum over the rows is a chain over its own registers,
// and the two halves of the wavefront are combined once at the end.
//
// The residual comes from an instance-major copy rT[R][m64] (made before each launch, rows
// padded to a multiple of 64 with zeros) so that the 32 residuals of a lane are 8 aligned
// 16-byte loads.
#include "dmmv_common.h"

namespace dmmv {

namespace {

typedef __attribute__((__vector_size__(32 * sizeof(float)))) float floatx32;

template <class T>
__global__ void k_transpose_pad(const T* __restrict__ in, int64_t rows, int64_t cols, int64_t ld_in,
                                T* __restrict__ out, int64_t ld_out) {
    // out[c][r] = in[r][c]
    __shared__ T tile[32][33];
    const int64_t c0 = blockIdx.x * 32ll, r0 = blockIdx.y * 32ll;
    for (int dy = threadIdx.y; dy < 32; dy += blockDim.y) {
        const int64_t rr = r0 + dy, cc = c0 + threadIdx.x;
        if (rr < rows && cc < cols) tile[dy][threadIdx.x] = in[rr * ld_in + cc];
    }
    __syncthreads();
    for (int dy = threadIdx.y; dy < 32; dy += blockDim.y) {
        const int64_t cc = c0 + dy, rr = r0 + threadIdx.x;
        if (rr < rows && cc < cols) out[cc * ld_out + rr] = tile[threadIdx.x][dy];
    }
}

__global__ void k_fill_zero_f32(float* p, int64_t count) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < count; e += stride) p[e] = 0.0f;
}

// grid.x = group of 4 * (32 / NDP) instances (one wavefront takes 32 / NDP of them),
// grid.y = chunk of chunk_cols variables; a wavefront goes through its chunk CC columns at a time.
// NDP = values of D per instance, padded to a power of two.
// Two wavefronts per SIMD at least: with at most 256 registers per lane the compiler keeps the
// results of the matrix instruction in ordinary vector registers, where the maximum reads them
// directly.
template <int NDP, int CC>
__global__ __launch_bounds__(256, 2) void k_eval_batched_mfma(
    int64_t m, int64_t m64, int64_t n, int64_t R, int32_t nd, int32_t chunk_cols,
    const float* __restrict__ X, int64_t lda, const float* __restrict__ D,
    const int32_t* __restrict__ kidx, const float* __restrict__ scale, const float* __restrict__ rT,
    int32_t radius, const uint8_t* __restrict__ var_mask, const InstState<float>* __restrict__ st,
    float* __restrict__ scores, Partial<float>* __restrict__ part) {
    constexpr int IPW = 32 / NDP;
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int half = lane >> 5, jj = lane & 31;
    const int qi = jj / NDP, k = jj % NDP;
    const int64_t q = ((int64_t)blockIdx.x * 4 + w) * IPW + qi;
    const bool inst_ok = q < R;
    const int64_t qc = inst_ok ? q : R - 1;
    const int32_t kk = k < nd ? k : nd - 1;
    const float sc = scale[qc];
    const float Dk = D[kk];
    const bool skip = part && !scores && st[qc].done;       // stopped instances score nothing
    const bool useful = inst_ok && k < nd && !skip;
    const bool writer = inst_ok && half == 0 && k == 0;
    if (__ballot(useful) == 0ull) {
        if (part && writer) { Partial<float> e; e.s = 0.0f; e.c = -1; part[blockIdx.y * R + q] = e; }
        return;
    }
    const int64_t jbeg = blockIdx.y * (int64_t)chunk_cols;
    const int64_t jend = jbeg + chunk_cols < n ? jbeg + chunk_cols : n;
    const float* __restrict__ rq = rT + qc * m64;
    float bs = 0.0f;
    int64_t bc = -1;
    for (int64_t c0 = jbeg; c0 < jend; c0 += CC) {
        float delta[CC], acc[CC];
#pragma unroll
        for (int u = 0; u < CC; ++u) {
            const int64_t j = c0 + u < n ? c0 + u : n - 1;
            const int32_t kc = kidx[j * R + qc];
            delta[u] = (useful && c0 + u < jend) ? step_of(Dk, D[kc], sc) : 0.0f;
            acc[u] = 0.0f;
        }
        for (int64_t row0 = 0; row0 < m; row0 += 64) {
            floatx32 cr;
#pragma unroll
            for (int g = 0; g < 8; ++g) {
                const float4 v4 = *reinterpret_cast<const float4*>(rq + row0 + 32 * (g >> 2) + 8 * (g & 3) + 4 * half);
                cr[g * 4 + 0] = v4.x; cr[g * 4 + 1] = v4.y; cr[g * 4 + 2] = v4.z; cr[g * 4 + 3] = v4.w;
            }
            const int64_t arow = row0 + lane;
            const bool arow_ok = arow < m;
            const float* __restrict__ xa = X + (arow_ok ? arow : 0);
            // the CC column entries of this row tile are all loaded before the first product
            float av[CC];
#pragma unroll
            for (int u = 0; u < CC; ++u) {
                const int64_t j = c0 + u < n ? c0 + u : n - 1;
                av[u] = arow_ok ? xa[j * lda] : 0.0f;
            }
            // Software pipeline: the product of column u is started before the result of column
            // u - 1 is folded into its running maximum.  The scheduling fences keep the compiler
            // from starting more products at once (32 result registers each).
            floatx32 dprev = __builtin_amdgcn_mfma_f32_32x32x1f32(av[0], delta[0], cr, 0, 0, 0);
#pragma unroll
            for (int u = 1; u <= CC; ++u) {
                floatx32 dcur = dprev;
                if (u < CC) dcur = __builtin_amdgcn_mfma_f32_32x32x1f32(av[u], delta[u], cr, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                float mx = acc[u - 1];
#pragma unroll
                for (int v = 0; v < 32; v += 2) mx = dmmv_max(dmmv_max(mx, dmmv_abs(dprev[v])), dmmv_abs(dprev[v + 1]));
                acc[u - 1] = mx;
                dprev = dcur;
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int u = 0; u < CC; ++u) {
            float val = dmmv_max(acc[u], __shfl_xor(acc[u], 32, 64));       // the other 32 rows of every tile
            const int64_t j = c0 + u;
            if (useful && half == 0 && j < jend) {
                const int32_t kc = kidx[j * R + q];
                const bool var_ok = var_mask ? var_mask[q * n + j] != 0 : true;
                if (!cand_allowed(kc, k, radius, var_ok)) val = Limits<float>::inf();
                const int64_t cidx = j * (int64_t)nd + k;
                if (scores) scores[q * (n * (int64_t)nd) + cidx] = val;
                if (rec_less(val, cidx, bs, bc)) { bs = val; bc = cidx; }
            }
        }
    }
    if (part) {
        // arg-min over the NDP lanes of an instance (records sit in the lower half only)
#pragma unroll
        for (int off = 1; off < NDP; off <<= 1) {
            const float os = __shfl_xor(bs, off, 64);
            const int64_t oc = (int64_t)__shfl_xor((long long)bc, off, 64);
            if (rec_less(os, oc, bs, bc)) { bs = os; bc = oc; }
        }
        if (writer) { Partial<float> p; p.s = bc < 0 ? 0.0f : bs; p.c = bc; part[blockIdx.y * R + q] = p; }
    }
}

template <int NDP>
dmmv_status launch_ndp(Ctx* c, void* scores, bool want_partials) {
    constexpr int CC = 16;
    constexpr int IPW = 32 / NDP;
    const int64_t m64 = ceil_div(c->p.m, 64) * 64;
    dim3 grid((unsigned)ceil_div(c->p.R, 4 * IPW), (unsigned)c->n_partials);
    hipLaunchKernelGGL((k_eval_batched_mfma<NDP, CC>), grid, dim3(256), 0, c->stream, c->p.m, m64, c->p.n, c->p.R,
                       c->p.nd, c->chunk_cols, (const float*)c->p.A_dense, c->p.lda, (const float*)c->D_dev,
                       (const int32_t*)c->kidx, (const float*)c->scale_dev, (const float*)c->rT, c->o.radius,
                       c->o.var_mask, (const InstState<float>*)c->state, (float*)scores,
                       want_partials ? (Partial<float>*)c->partials : nullptr);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

}  // namespace

bool batched_eval_mfma_applicable(const dmmv_problem& p) {
    return p.dtype == DMMV_F32 && p.nd <= 32;
}

int64_t batched_eval_mfma_rt_elems(const dmmv_problem& p) { return p.R * (ceil_div(p.m, 64) * 64); }

// zero the instance-major residual copy once: its row padding must read as zero
dmmv_status batched_eval_mfma_build(Ctx* c) {
    const int64_t count = batched_eval_mfma_rt_elems(c->p);
    if (count == 0) return DMMV_OK;
    hipLaunchKernelGGL(k_fill_zero_f32, dim3(2048), dim3(256), 0, c->stream, (float*)c->rT, count);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

dmmv_status batched_eval_mfma(Ctx* c, void* scores, bool want_partials) {
    const int64_t m = c->p.m, R = c->p.R;
    if (c->p.n == 0 || R == 0) return DMMV_OK;
    if ((c->chunk_cols & 31) != 0) return fail(DMMV_ERR_STATE, "batched evaluation: chunk of %d columns is not a multiple of 32", c->chunk_cols);
    const int64_t m64 = ceil_div(m, 64) * 64;
    if (m > 0) {
        // r [m][R] -> rT [R][m64]
        dim3 grid((unsigned)ceil_div(R, 32), (unsigned)ceil_div(m, 32));
        hipLaunchKernelGGL(k_transpose_pad<float>, grid, dim3(32, 8), 0, c->stream, (const float*)c->r, m, R, R,
                           (float*)c->rT, m64);
    }
    const int32_t nd = c->p.nd;
    if (nd <= 2) return launch_ndp<2>(c, scores, want_partials);
    if (nd <= 4) return launch_ndp<4>(c, scores, want_partials);
    if (nd <= 8) return launch_ndp<8>(c, scores, want_partials);
    if (nd <= 16) return launch_ndp<16>(c, scores, want_partials);
    return launch_ndp<32>(c, scores, want_partials);
}

}  // namespace dmmv
