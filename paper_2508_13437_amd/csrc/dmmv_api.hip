// C ABI of libdmmv: validation, workspace layout, call sequencing, and the small kernels
// shared by the three storage kinds (value<->index conversion, selection of the best move
// from partial records, arg-min of a given table, max |r|).
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <new>
#include <utility>
#include <vector>

#include "dmmv_common.h"
#include "../../include/dmmv_bench.h"

namespace dmmv {

// ----------------------------------------------------------------------------------------
// errors
// ----------------------------------------------------------------------------------------
static thread_local char g_err[512] = "";

dmmv_status fail(dmmv_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

// The attribute belongs to the kernel ON ONE DEVICE, so what has been done is remembered per
// (device, kernel); the list stays short (a few kernels per device).
dmmv_status ensure_dynamic_lds(const void* kernel, int bytes) {
    static std::mutex mu;
    static std::vector<std::pair<int, const void*>> done;
    int dev = -1;
    DMMV_HIP_CHECK(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(mu);
    for (const auto& e : done)
        if (e.first == dev && e.second == kernel) return DMMV_OK;
    DMMV_HIP_CHECK(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    done.emplace_back(dev, kernel);
    return DMMV_OK;
}

// ----------------------------------------------------------------------------------------
// workspace layout
// ----------------------------------------------------------------------------------------
namespace {
struct Bump {
    char* base;
    size_t off = 0;
    template <class P>
    void take(P** out, size_t bytes) {
        off = (off + 255) / 256 * 256;
        if (out) *out = base ? reinterpret_cast<P*>(base + off) : nullptr;
        off += bytes;
    }
};

}  // namespace

int32_t batched_chunk_cols(const dmmv_problem& p) {
    // 512 workgroups are resident at a time (2 per CU), each for the whole of its chunk: aim at
    // some 30 rounds of them so that the last, partly filled round costs a few percent at most
    int64_t groups = ceil_div(p.R, 64);
    int64_t want_chunks = ceil_div(16384, groups);
    int64_t cols = ceil_div(p.n, want_chunks);
    cols = ceil_div(cols, 32) * 32;
    if (cols < 32) cols = 32;
    return (int32_t)cols;
}

// sparse matrices: rows per LDS-resident partition of r (what fits the LDS budget, addressable by
// a 16-bit offset) and the number of partitions
static void sparse_partitions(const dmmv_problem& p, const dmmv_options& o, int64_t* mp_out, int64_t* P_out) {
    const int64_t esz = p.dtype == DMMV_F64 ? 8 : 4;
    int64_t mp = o.sparse_partition_rows > 0 ? o.sparse_partition_rows : (int64_t)(CSC_LDS_BYTES / esz);
    if (mp > 65535) mp = 65535;          // offset mp itself marks a pad
    if (mp * esz > CSC_LDS_BYTES) mp = CSC_LDS_BYTES / esz;
    *mp_out = mp;
    *P_out = p.m > 0 ? ceil_div(p.m, mp) : 1;
}

size_t workspace_layout(const dmmv_problem& p, const dmmv_options& o, Ctx* c, char* base) {
    (void)o;
    Ctx dummy;
    if (!c) c = &dummy;
    const size_t esz = p.dtype == DMMV_F64 ? 8 : 4;
    const bool sparse = p.csr_rowptr != nullptr;
    const bool batched = !sparse && (p.R > 1 || p.scale != nullptr);
    const size_t state_sz = p.dtype == DMMV_F64 ? sizeof(InstState<double>) : sizeof(InstState<float>);
    const size_t part_sz = p.dtype == DMMV_F64 ? sizeof(Partial<double>) : sizeof(Partial<float>);
    Bump b{base};
    b.take(&c->flags, FLAG_COUNT * sizeof(int32_t));
    b.take(&c->D_dev, (size_t)p.nd * esz);
    b.take(&c->scale_dev, (size_t)p.R * esz);
    b.take(&c->state, (size_t)p.R * state_sz);
    b.take(&c->kidx, (size_t)p.n * p.R * sizeof(int32_t));
    b.take(&c->r, (size_t)p.m * p.R * esz);
    c->red_elems = 1024;
    b.take(&c->red, (size_t)c->red_elems * esz);
    if (!batched || o.alns) {
        // ALNS outer loop: current and best solution, sampling weights, draws (per instance)
        const size_t nR = (size_t)p.n * p.R, mR = (size_t)p.m * p.R;
        b.take(&c->alns_state, (size_t)p.R * sizeof(AlnsState));
        b.take(&c->alns_kidx_cur, nR * sizeof(int32_t));
        b.take(&c->alns_kidx_best, nR * sizeof(int32_t));
        b.take(&c->alns_r_cur, mR * esz);
        b.take(&c->alns_weight, nR * sizeof(uint64_t));
        b.take(&c->alns_prefix, nR * sizeof(uint64_t));
        b.take(&c->alns_first, nR * sizeof(uint64_t));
        b.take(&c->alns_picked, nR * sizeof(int32_t));
        if (sparse) {
            b.take(&c->alns_touched, (size_t)p.m);
            b.take(&c->alns_g_row, ((size_t)1 << 20) * sizeof(int32_t));
            b.take(&c->alns_g_val, ((size_t)1 << 20) * esz);
        }
        b.take(&c->alns_q2, (size_t)p.R * sizeof(double));
        b.take(&c->alns_q2_blocks, (size_t)(ceil_div(p.m, 256) + 1) * sizeof(double));
    }
    if (o.l2_rule) {
        b.take(&c->l2_g, (size_t)p.n * p.R * esz);
        b.take(&c->l2_c, (size_t)p.n * esz);
        if (o.l2_rule != 3) b.take(&c->l2_scores, (size_t)p.n * p.R * p.nd * esz);
    }
    if (!sparse && !batched) b.take(&c->persist_exchange, dense_persistent_exchange_bytes());
    if (!sparse) {
        c->swap_nb = swap_blocks_per_instance(p);
        b.take(&c->swap_rows, (size_t)p.R * SWAP_KMAX * sizeof(int32_t));
        b.take(&c->swap_part, (size_t)p.R * c->swap_nb * part_sz);
        b.take(&c->swap_skip, (size_t)p.R * sizeof(int32_t));
    }
    if (sparse) {
        int64_t mp, P;
        sparse_partitions(p, o, &mp, &P);
        c->csc_mp = (int32_t)mp;
        c->csc_P = (int32_t)P;
        int64_t gb = 512 / c->csc_P;         // about two workgroups per compute unit in all
        if (gb > ceil_div(p.n, 16)) gb = ceil_div(p.n, 16);
        if (gb < 1) gb = 1;
        c->csc_gb = (int32_t)gb;
        // One-kernel evaluation: each of its ceil(n / 256) workgroups reads all of r, so it is
        // taken when that traffic does not exceed the matrix itself (about w + 2 bytes an entry)
        {
            const double r_traffic = (double)ceil_div(p.n, 256) * (double)p.m * (double)esz;
            const double a_traffic = ((double)p.nnz + 2.0 * (double)c->csc_P * (double)p.n) * (double)(esz + 2);
            // (fp64: its registers do not fit without spills, the two-kernel path is the faster one)
            c->csc_fused = c->csc_P <= 16 && (o.sparse_eval == 2 || (o.sparse_eval == 0 && p.dtype == DMMV_F32 && r_traffic <= a_traffic));
        }
        const int64_t nseg = (int64_t)c->csc_P * p.n;
        c->csc_nnzp = p.nnz + 4 * nseg + 4;  // padding bound (an empty segment holds four pads), plus spare entries
        c->n_partials = ceil_div(p.n, CSC_FIN_BLOCK);
        b.take(&c->partials, (size_t)(c->n_partials > 0 ? c->n_partials : 1) * part_sz);
        b.take(&c->segptr, (size_t)(nseg + 1) * sizeof(int32_t));
        b.take(&c->fillpos, (size_t)(nseg + 1) * sizeof(int32_t));
        b.take(&c->row16, (size_t)c->csc_nnzp * sizeof(uint16_t));
        b.take(&c->cval, (size_t)c->csc_nnzp * esz);
        b.take(&c->row16_tmp, (size_t)c->csc_nnzp * sizeof(uint16_t));
        b.take(&c->cval_tmp, (size_t)c->csc_nnzp * esz);
        b.take(&c->blk_lo, (size_t)c->csc_P * (gb + 1) * sizeof(int32_t));
        b.take(&c->part_scores, (size_t)nseg * p.nd * esz);
        b.take(&c->part_mask, (size_t)nseg * sizeof(uint32_t));
        b.take(&c->res_val, (size_t)RES_CAP * esz);
        b.take(&c->res_row, (size_t)RES_CAP * sizeof(int32_t));
        b.take(&c->res_meta, 4 * sizeof(int32_t));
        b.take(&c->res_floor, esz);
        if (o.prune) b.take(&c->prune_part, (size_t)(p.n > 0 ? p.n : 1) * part_sz);
        b.take(&c->swap_part, (size_t)swap_csc_records(p) * part_sz);
        b.take(&c->swap_skip, sizeof(int32_t));
        b.take(&c->swap_gbest, sizeof(unsigned long long));
    } else if (batched) {
        c->chunk_cols = batched_chunk_cols(p);
        c->n_partials = ceil_div(p.n, c->chunk_cols);
        b.take(&c->partials, (size_t)(c->n_partials > 0 ? c->n_partials : 1) * p.R * part_sz);
        b.take(&c->Xt, (size_t)p.m * p.n * esz);
        b.take(&c->Bt, (size_t)p.m * p.R * esz);
        b.take(&c->cmp_r, (size_t)p.m * p.R * esz);
        b.take(&c->cmp_kidx, (size_t)p.n * p.R * sizeof(int32_t));
        b.take(&c->cmp_state, (size_t)p.R * state_sz);
        b.take(&c->cmp_scale, (size_t)p.R * esz);
        b.take(&c->cmp_orig, (size_t)p.R * sizeof(int32_t));
        c->eval_mfma = o.batched_eval == 2 && batched_eval_mfma_applicable(p);
        if (c->eval_mfma) b.take(&c->rT, (size_t)batched_eval_mfma_rt_elems(p) * sizeof(float));
        if (o.residual_mfma) {
            c->mfma_ldk = mfma_ldk(p.n);
            b.take(&c->Xp, (size_t)3 * p.m * c->mfma_ldk * sizeof(uint16_t));
            b.take(&c->Qt, (size_t)p.R * c->mfma_ldk * sizeof(uint16_t));
        }
    } else {
        c->n_partials = dense_num_partials(p);
        b.take(&c->partials, (size_t)(c->n_partials > 0 ? c->n_partials : 1) * part_sz);
        if (o.value_search) b.take(&c->search_part, (size_t)(p.n > 0 ? p.n : 1) * part_sz);
        if (o.prune) b.take(&c->Xt, (size_t)p.m * p.n * esz);     // the pruned descent reads rows of A
    }
    return (b.off + 255) / 256 * 256;
}

// ----------------------------------------------------------------------------------------
// validation (host)
// ----------------------------------------------------------------------------------------
static dmmv_status validate_problem(const dmmv_problem* p) {
    if (!p) return fail(DMMV_ERR_NULL, "problem is NULL");
    if (p->dtype != DMMV_F32 && p->dtype != DMMV_F64) return fail(DMMV_ERR_DTYPE, "dtype %d is not DMMV_F32/DMMV_F64", p->dtype);
    if (p->m < 0 || p->n < 0 || p->R < 1) return fail(DMMV_ERR_SHAPE, "need m >= 0, n >= 0, R >= 1 (m=%lld n=%lld R=%lld)", (long long)p->m, (long long)p->n, (long long)p->R);
    if (p->m > INT32_MAX - 1 || p->n > INT32_MAX - 1) return fail(DMMV_ERR_SHAPE, "m and n must fit in 31 bits");
    if (p->nd < 2 || p->nd > 65535) return fail(DMMV_ERR_DOMAIN, "need 2 <= nd <= 65535 (nd=%d)", p->nd);
    if (!p->D) return fail(DMMV_ERR_NULL, "D is NULL");
    for (int32_t k = 0; k < p->nd; ++k) {
        double v = p->dtype == DMMV_F64 ? ((const double*)p->D)[k] : (double)((const float*)p->D)[k];
        if (!isfinite(v)) return fail(DMMV_ERR_DOMAIN, "D[%d] is not finite", k);
        if (k > 0) {
            double u = p->dtype == DMMV_F64 ? ((const double*)p->D)[k - 1] : (double)((const float*)p->D)[k - 1];
            if (!(u < v)) return fail(DMMV_ERR_DOMAIN, "D is not strictly ascending at index %d", k);
        }
    }
    const bool dense = p->A_dense != nullptr;
    const bool sparse = p->csr_rowptr != nullptr;
    if (dense == sparse && (p->m > 0 && p->n > 0)) return fail(DMMV_ERR_NULL, "exactly one of A_dense and csr_rowptr must be set");
    if (dense && p->lda < (p->m > 1 ? p->m : 1)) return fail(DMMV_ERR_SHAPE, "lda=%lld < max(m,1)", (long long)p->lda);
    if (sparse) {
        if (p->nnz < 0 || p->nnz > INT32_MAX - 1) return fail(DMMV_ERR_SHAPE, "nnz must be in [0, 2^31-2]");
        if (p->nnz > 0 && (!p->csr_col || !p->csr_val)) return fail(DMMV_ERR_NULL, "csr_col / csr_val is NULL");
        if (p->R != 1 || p->scale) return fail(DMMV_ERR_UNSUPPORTED, "sparse matrices support a single unscaled instance (R = 1, scale = NULL)");
    }
    if (p->m > 0 && !p->b) return fail(DMMV_ERR_NULL, "b is NULL");
    if (p->scale) {
        for (int64_t q = 0; q < p->R; ++q) {
            double v = p->dtype == DMMV_F64 ? ((const double*)p->scale)[q] : (double)((const float*)p->scale)[q];
            if (!isfinite(v) || !(v > 0)) return fail(DMMV_ERR_DOMAIN, "scale[%lld] must be finite and positive", (long long)q);
        }
    } else if (p->R != 1) {
        return fail(DMMV_ERR_NULL, "scale is NULL but R = %lld", (long long)p->R);
    }
    return DMMV_OK;
}

// ----------------------------------------------------------------------------------------
// shared kernels
// ----------------------------------------------------------------------------------------
template <class T>
__global__ void k_init_state(InstState<T>* st, int64_t R) {
    int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q >= R) return;
    InstState<T> s;
    s.t = (T)0; s.best_s = (T)0; s.delta = (T)0;
    s.apply_j = -1; s.apply_k = -1; s.done = 0; s.moves = 0;
    st[q] = s;
}

__global__ void k_zero_flags(int32_t* flags) {
    if (threadIdx.x < FLAG_COUNT) flags[threadIdx.x] = 0;
}

// x values -> index into D (binary search, exact match required), single instance
template <class T>
__global__ void k_values_to_index(const T* __restrict__ x, const T* __restrict__ D, int32_t nd,
                                  int64_t n, int32_t* __restrict__ kidx, int32_t* flags) {
    int64_t j = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (j >= n) return;
    T v = x[j];
    int32_t lo = 0, hi = nd - 1;
    while (lo < hi) {
        int32_t mid = (lo + hi) >> 1;
        if (D[mid] < v) lo = mid + 1; else hi = mid;
    }
    if (!(D[lo] == v)) { atomicOr(&flags[FLAG_ERROR], ERRBIT_X_NOT_IN_D); lo = 0; }
    kidx[j] = lo;
}

template <class T>
__global__ void k_index_to_values(const int32_t* __restrict__ kidx, const T* __restrict__ D,
                                  int64_t n, T* __restrict__ x) {
    int64_t j = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (j < n) x[j] = D[kidx[j]];
}

// stage 1 of max |r|: one partial per block
template <class T>
__global__ void k_maxabs_partial(const T* __restrict__ r, int64_t m, T* __restrict__ red) {
    __shared__ T sh[16];
    T v = (T)0;
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < m;
         i += (int64_t)gridDim.x * blockDim.x)
        v = dmmv_max(v, dmmv_abs(r[i]));
    v = wave_max(v);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        T w = (T)0;
        for (int q = 0; q < (int)(blockDim.x >> 6); ++q) w = dmmv_max(w, sh[q]);
        red[blockIdx.x] = w;
    }
}

template <class T>
__global__ void k_maxabs_final(const T* __restrict__ red, int nred, InstState<T>* st) {
    T v = (T)0;
    for (int q = threadIdx.x; q < nred; q += blockDim.x) v = dmmv_max(v, red[q]);
    v = wave_max(v);
    __shared__ T sh[16];
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        T w = (T)0;
        for (int q = 0; q < (int)(blockDim.x >> 6); ++q) w = dmmv_max(w, sh[q]);
        st[0].t = w;
    }
}

// Selection for a single instance: reduce the partial records of the fused evaluation to the
// best move, decide whether it is a strict improvement and stage it for the apply kernel.
template <class T>
__global__ void k_select_single(const Partial<T>* __restrict__ part, int64_t n_part,
                                InstState<T>* st, const T* __restrict__ D,
                                const int32_t* __restrict__ kidx, int32_t nd, int32_t keep_going,
                                dmmv_move* best_out, T* best_score_out) {
    __shared__ T sh_s[16];
    __shared__ int64_t sh_c[16];
    if (st[0].done && !best_out) return;
    T s = (T)0;
    int64_t c = -1;
    for (int64_t q = threadIdx.x; q < n_part; q += blockDim.x) {
        Partial<T> p = part[q];
        if (rec_less(p.s, p.c, s, c)) { s = p.s; c = p.c; }
    }
    block_argmin(s, c, sh_s, sh_c);
    if (threadIdx.x == 0) {
        InstState<T> z = st[0];
        int32_t j = -1, k = -1;
        if (c >= 0) { j = (int32_t)(c / nd); k = (int32_t)(c % nd); }
        const bool improving = c >= 0 && s < z.t;
        z.best_s = s;
        z.apply_j = improving ? j : -1;
        z.apply_k = improving ? k : -1;
        z.delta = improving ? step_of(D[k], D[kidx[j]], (T)1) : (T)0;
        if (!improving && !keep_going) z.done = 1;
        st[0] = z;
        if (best_out) { best_out[0].j = j; best_out[0].k = k; }
        if (best_score_out) best_score_out[0] = c >= 0 ? s : Limits<T>::inf();
    }
}

// Same for a batch: one lane per instance, partial records laid out [chunk][R].
template <class T>
__global__ void k_select_batched(const Partial<T>* __restrict__ part, int64_t n_part, int64_t R,
                                 InstState<T>* st, const T* __restrict__ D,
                                 const T* __restrict__ scale, const int32_t* __restrict__ kidx,
                                 int32_t nd, int32_t keep_going, dmmv_move* best_out,
                                 T* best_score_out) {
    int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q >= R) return;
    InstState<T> z = st[q];
    if (z.done && !best_out) return;
    T s = (T)0;
    int64_t c = -1;
    for (int64_t ch = 0; ch < n_part; ++ch) {
        Partial<T> p = part[ch * R + q];
        if (rec_less(p.s, p.c, s, c)) { s = p.s; c = p.c; }
    }
    int32_t j = -1, k = -1;
    if (c >= 0) { j = (int32_t)(c / nd); k = (int32_t)(c % nd); }
    const bool improving = c >= 0 && s < z.t;
    z.best_s = s;
    z.apply_j = improving ? j : -1;
    z.apply_k = improving ? k : -1;
    z.delta = improving ? step_of(D[k], D[kidx[(int64_t)j * R + q]], scale[q]) : (T)0;
    if (!improving && !keep_going) z.done = 1;
    st[q] = z;
    if (best_out) { best_out[q].j = j; best_out[q].k = k; }
    if (best_score_out) best_score_out[q] = c >= 0 ? s : Limits<T>::inf();
}

// Arg-min of a caller-supplied table, one block per instance.
template <class T>
__global__ void k_argmin_table(const T* __restrict__ scores, int64_t ntab, int32_t nd,
                               dmmv_move* best_out, T* best_score_out) {
    __shared__ T sh_s[16];
    __shared__ int64_t sh_c[16];
    const int64_t q = blockIdx.x;
    const T* tab = scores + q * ntab;
    T s = (T)0;
    int64_t c = -1;
    for (int64_t i = threadIdx.x; i < ntab; i += blockDim.x) {
        T v = tab[i];
        if (rec_less(v, i, s, c)) { s = v; c = i; }
    }
    block_argmin(s, c, sh_s, sh_c);
    if (threadIdx.x == 0) {
        if (best_out) {
            best_out[q].j = c >= 0 ? (int32_t)(c / nd) : -1;
            best_out[q].k = c >= 0 ? (int32_t)(c % nd) : -1;
        }
        if (best_score_out) best_score_out[q] = c >= 0 ? s : Limits<T>::inf();
    }
}

// Stage caller-supplied moves for the apply kernels (dmmv_apply_move).
template <class T>
__global__ void k_stage_moves(const dmmv_move* __restrict__ moves, int64_t R, int64_t n,
                              int32_t nd, InstState<T>* st, const T* __restrict__ D,
                              const T* __restrict__ scale, const int32_t* __restrict__ kidx,
                              int32_t* flags) {
    int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q >= R) return;
    dmmv_move mv = moves[q];
    InstState<T> z = st[q];
    z.apply_j = -1; z.apply_k = -1; z.delta = (T)0;
    if (mv.j >= 0) {
        if (mv.j >= n || mv.k < 0 || mv.k >= nd) {
            atomicOr(&flags[FLAG_ERROR], ERRBIT_MOVE_RANGE);
        } else {
            z.apply_j = mv.j; z.apply_k = mv.k;
            z.delta = step_of(D[mv.k], D[kidx[(int64_t)mv.j * R + q]], scale ? scale[q] : (T)1);
        }
    }
    st[q] = z;
}

template <class T>
__global__ void k_count_active(const InstState<T>* __restrict__ st, int64_t R, int32_t* flags) {
    int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q < R && !st[q].done) atomicAdd(&flags[FLAG_ACTIVE], 1);
}

// a stopped instance is skipped by the fused evaluation; standalone queries clear the mark
template <class T>
__global__ void k_clear_done(InstState<T>* st, int64_t R) {
    int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q < R) st[q].done = 0;
}

template <class T>
__global__ void k_reset_loop(InstState<T>* st, int64_t R) {
    int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q < R) { st[q].done = 0; st[q].moves = 0; st[q].apply_j = -1; }
}

template <class T>
__global__ void k_fill_trace(dmmv_move* trace, T* trace_t, int64_t count) {
    int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q >= count) return;
    if (trace) { trace[q].j = -1; trace[q].k = -1; }
    if (trace_t) trace_t[q] = (T)0;
}

template <class T>
__global__ void k_export_state(const InstState<T>* __restrict__ st, int64_t R, T* t_out,
                               int32_t* moves_out) {
    int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q >= R) return;
    if (t_out) t_out[q] = st[q].t;
    if (moves_out) moves_out[q] = st[q].moves;
}

static inline dim3 grid1(int64_t n, int block) { return dim3((unsigned)(n > 0 ? ceil_div(n, block) : 1)); }

template <class T>
static dmmv_status maxabs_single(Ctx* c) {
    const int nblk = (int)(c->p.m > 0 ? (ceil_div(c->p.m, 1024) < c->red_elems ? ceil_div(c->p.m, 1024) : c->red_elems) : 1);
    hipLaunchKernelGGL(k_maxabs_partial<T>, dim3(nblk), dim3(256), 0, c->stream, (const T*)c->r, c->p.m, (T*)c->red);
    hipLaunchKernelGGL(k_maxabs_final<T>, dim3(1), dim3(256), 0, c->stream, (const T*)c->red, nblk, (InstState<T>*)c->state);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

// t = max |r| into the state, whatever the kind
// (sparse: also rebuilds the reservoir of the rows of largest |r|)
static dmmv_status refresh_t(Ctx* c) {
    if (c->kind == KIND_BATCHED) return batched_maxabs(c);
    if (c->kind == KIND_CSC) DMMV_TRY(csc_reservoir(c));
    return c->p.dtype == DMMV_F64 ? maxabs_single<double>(c) : maxabs_single<float>(c);
}

template <class T>
static dmmv_status select_t(Ctx* c, dmmv_move* best_out, void* best_score_out) {
    if (c->kind == KIND_BATCHED) {
        hipLaunchKernelGGL(k_select_batched<T>, grid1(c->p.R, 256), dim3(256), 0, c->stream,
                           (const Partial<T>*)c->partials, c->p.n > 0 ? c->n_partials : 0, c->p.R,
                           (InstState<T>*)c->state, (const T*)c->D_dev, (const T*)c->scale_dev,
                           (const int32_t*)c->kidx, c->p.nd, c->o.keep_going, best_out,
                           (T*)best_score_out);
    } else {
        hipLaunchKernelGGL(k_select_single<T>, dim3(1), dim3(1024), 0, c->stream,
                           (const Partial<T>*)c->partials, c->p.n > 0 ? c->n_partials : 0,
                           (InstState<T>*)c->state, (const T*)c->D_dev, (const int32_t*)c->kidx,
                           c->p.nd, c->o.keep_going, best_out, (T*)best_score_out);
    }
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}
static dmmv_status launch_select(Ctx* c, dmmv_move* best_out, void* best_score_out) {
    return c->p.dtype == DMMV_F64 ? select_t<double>(c, best_out, best_score_out)
                                  : select_t<float>(c, best_out, best_score_out);
}

static dmmv_status eval_any(Ctx* c, void* scores_out, bool want_partials, bool honor_done) {
    if (c->p.n == 0) return DMMV_OK;
    switch (c->kind) {
        case KIND_DENSE: return dense_eval(c, scores_out, want_partials, honor_done);
        case KIND_CSC:
            return csc_eval(c, scores_out, want_partials, honor_done);
        default: return batched_eval(c, scores_out, want_partials);
    }
}

static dmmv_status apply_any(Ctx* c, bool t_from_score, int32_t iters, dmmv_move* trace, void* trace_t) {
    switch (c->kind) {
        case KIND_DENSE: return dense_apply(c, t_from_score, iters, trace, trace_t);
        case KIND_CSC: return csc_apply(c);   // staged moves only; the loop uses csc_select_apply
        default: return batched_apply(c, t_from_score, iters, trace, trace_t);
    }
}

// One step of the descent.  Sparse matrices with options.prune (and not in fixed-work mode)
// score only the columns that touch the row of largest |r|: same moves, far less work.
static dmmv_status loop_step(Ctx* c, int32_t iters, dmmv_move* trace, void* trace_t);

// one loop step after the evaluation: pick the best move and apply it if it improves
static dmmv_status select_apply_any(Ctx* c, int32_t iters, dmmv_move* trace, void* trace_t) {
    if (c->kind == KIND_CSC) return csc_select_apply(c, iters, trace, trace_t, false);
    if (c->kind == KIND_DENSE && dense_has_fused_select_apply(c)) return dense_select_apply(c, iters, trace, trace_t);
    DMMV_TRY(launch_select(c, nullptr, nullptr));
    return apply_any(c, true, iters, trace, trace_t);
}

// One step with the l2 change as second criterion: the evaluation writes the whole score table,
// g = A^T r follows the residual, the selection reads both.  (The exact prunings drop candidates
// that cannot win on the score alone, so they do not apply here.)
static dmmv_status loop_step_l2(Ctx* c, int32_t iters, dmmv_move* trace, void* trace_t) {
    if (c->p.n == 0) return DMMV_OK;
    DMMV_TRY(eval_any(c, c->l2_scores, false, true));
    DMMV_TRY(l2_update_g(c));
    DMMV_TRY(l2_select(c, c->l2_scores, c->o.keep_going, nullptr, nullptr));
    if (c->kind != KIND_CSC) return apply_any(c, true, iters, trace, trace_t);
    DMMV_TRY(csc_apply(c));
    DMMV_TRY(l2_after_apply_csc(c, iters, trace, trace_t));
    return csc_reservoir(c);
}

static dmmv_status loop_step(Ctx* c, int32_t iters, dmmv_move* trace, void* trace_t) {
    if (c->o.l2_rule == 1 || c->o.l2_rule == 2) return loop_step_l2(c, iters, trace, trace_t);
    if (batched_pruned_applicable(c)) return batched_descent_pruned(c, 1, iters, trace, trace_t);
    if (c->kind == KIND_CSC && c->o.prune && !c->o.keep_going && c->p.n > 0) {
        DMMV_TRY(csc_eval_pruned(c, true));
        return csc_select_apply(c, iters, trace, trace_t, true);
    }
    if (c->kind == KIND_DENSE && c->o.value_search && !c->o.keep_going && c->p.n > 0) {
        // one record per variable instead of one per evaluation workgroup
        DMMV_TRY(dense_eval_search(c, true));
        void* const part = c->partials;
        const int64_t n_part = c->n_partials;
        c->partials = c->search_part;
        c->n_partials = c->p.n;
        const dmmv_status st = select_apply_any(c, iters, trace, trace_t);
        c->partials = part;
        c->n_partials = n_part;
        return st;
    }
    DMMV_TRY(eval_any(c, nullptr, true, true));
    return select_apply_any(c, iters, trace, trace_t);
}

static dmmv_status residual_any(Ctx* c) {
    switch (c->kind) {
        case KIND_DENSE: DMMV_TRY(dense_residual(c)); break;
        case KIND_CSC: DMMV_TRY(csc_residual(c)); break;
        default:
            if (c->o.residual_mfma) DMMV_TRY(batched_mfma_residual(c));
            else DMMV_TRY(batched_residual(c));
            break;
    }
    DMMV_TRY(refresh_t(c));
    c->r_valid = true;
    return DMMV_OK;
}

// read and clear the device error flag (waits for the stream)
static dmmv_status check_device_errors(Ctx* c, int32_t* raw = nullptr) {
    int32_t host_flag = 0;
    DMMV_HIP_CHECK(hipMemcpyAsync(&host_flag, &c->flags[FLAG_ERROR], sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    DMMV_HIP_CHECK(hipStreamSynchronize(c->stream));
    if (raw) *raw = host_flag;
    if (host_flag) {
        hipLaunchKernelGGL(k_zero_flags, dim3(1), dim3(64), 0, c->stream, c->flags);
        DMMV_HIP_CHECK(hipStreamSynchronize(c->stream));
        if (host_flag & ERRBIT_X_NOT_IN_D) return fail(DMMV_ERR_DOMAIN, "x has a value that is not an element of D");
        if (host_flag & ERRBIT_CSR_RANGE) return fail(DMMV_ERR_SHAPE, "CSR column index out of range or row pointers not ascending");
        if (host_flag & ERRBIT_CSR_DUP) return fail(DMMV_ERR_SHAPE, "CSR matrix stores the same (row, column) entry twice");
        if (host_flag & ERRBIT_MOVE_RANGE) return fail(DMMV_ERR_SHAPE, "move with j >= n or k outside [0, nd)");
        if (host_flag & ERRBIT_WAIT_LIMIT)
            return fail(DMMV_ERR_STATE, "one-launch descent: a workgroup waited options.wait_limit polls for another one "
                        "(is another kernel holding compute units?); the state is that of the starting point");
        return fail(DMMV_ERR_STATE, "device error flag %d", host_flag);
    }
    return DMMV_OK;
}

template <class T>
static dmmv_status set_x_single(Ctx* c, const void* x) {
    hipLaunchKernelGGL(k_values_to_index<T>, grid1(c->p.n, 256), dim3(256), 0, c->stream,
                       (const T*)x, (const T*)c->D_dev, c->p.nd, c->p.n, c->kidx, c->flags);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status solve_t(dmmv_ctx* c, const void* x0, int32_t iters, void* x_out, void* t_out,
                           int32_t* iters_done, dmmv_move* trace, void* trace_t) {
    const int64_t R = c->p.R;
    if (x0 || c->p.n == 0) DMMV_TRY(dmmv_set_x(c, x0));
    if (!c->x_set) return fail(DMMV_ERR_STATE, "dmmv_solve: no starting point (x0 is NULL and dmmv_set_x was never called)");
    hipLaunchKernelGGL(k_reset_loop<T>, grid1(R, 256), dim3(256), 0, c->stream, (InstState<T>*)c->state, R);
    DMMV_TRY(residual_any(c));
    if (iters > 0 && (trace || trace_t))
        hipLaunchKernelGGL(k_fill_trace<T>, grid1(R * (int64_t)iters, 256), dim3(256), 0, c->stream, trace, (T*)trace_t, R * (int64_t)iters);
    int32_t poll = c->o.keep_going ? 0 : c->o.poll_every;
    // a batch drops its stopped instances at the polling points (their wavefronts would
    // otherwise keep running for the sake of a few neighbours), so it polls more often
    const bool pruned_batch = batched_pruned_applicable(c);
    const bool l2_on = c->o.l2_rule == 1 || c->o.l2_rule == 2;
    const bool compacting = c->kind == KIND_BATCHED && poll > 0 && !c->o.var_mask && !pruned_batch && !l2_on;
    if (compacting && poll > 8) poll = 8;
    dmmv_status loop_st = [&]() -> dmmv_status {
        // a pruned batch runs all its iterations in one launch; every instance stops by itself
        if (pruned_batch) return batched_descent_pruned(c, iters, iters, trace, trace_t);
        // a small dense instance too; the wait between its workgroups is bounded and reports here
        if (iters > 0 && dense_persistent_applicable(c)) {
            DMMV_TRY(dense_descent_persistent(c, iters, trace, trace_t));
            int32_t raw = 0;
            const dmmv_status one = check_device_errors(c, &raw);
            // An automatic choice must not add a way to fail: if the workgroups could not all be
            // resident (the device is shared), the attempt has left x, r and the loop state alone,
            // and the loop of launches below does the same descent.
            if (!(one != DMMV_OK && raw == ERRBIT_WAIT_LIMIT && c->o.dense_loop == 0)) return one;
            if (trace || trace_t)
                hipLaunchKernelGGL(k_fill_trace<T>, grid1(R * (int64_t)iters, 256), dim3(256), 0, c->stream, trace, (T*)trace_t, R * (int64_t)iters);
        }
        for (int32_t it = 0; it < iters; ++it) {
            DMMV_TRY(loop_step(c, iters, trace, trace_t));
            if (poll > 0 && (it + 1) % poll == 0 && it + 1 < iters) {
                int32_t active = 0;
                if (compacting) {
                    DMMV_TRY(batched_compact(c, &active));
                } else {
                    hipLaunchKernelGGL(k_zero_flags, dim3(1), dim3(64), 0, c->stream, c->flags);
                    hipLaunchKernelGGL(k_count_active<T>, grid1(R, 256), dim3(256), 0, c->stream, (const InstState<T>*)c->state, R, c->flags);
                    DMMV_HIP_CHECK(hipMemcpyAsync(&active, &c->flags[FLAG_ACTIVE], sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
                    DMMV_HIP_CHECK(hipStreamSynchronize(c->stream));
                }
                if (active == 0) break;
            }
        }
        return DMMV_OK;
    }();
    if (compacting) {
        const dmmv_status back = batched_compact_end(c);
        if (loop_st == DMMV_OK) loop_st = back;
    }
    DMMV_TRY(loop_st);
    hipLaunchKernelGGL(k_export_state<T>, grid1(R, 256), dim3(256), 0, c->stream, (const InstState<T>*)c->state, R, (T*)t_out, iters_done);
    DMMV_LAUNCH_CHECK();
    if (x_out) DMMV_TRY(dmmv_get_state(c, x_out, nullptr, nullptr));
    DMMV_HIP_CHECK(hipStreamSynchronize(c->stream));
    return DMMV_OK;
}

// ---- ALNS outer loop (Algorithm 1): destroy + repair, local search, accept ---------------
static dmmv_status alns_run(dmmv_ctx* c, const void* x0, const dmmv_alns_params& prm, void* x_best_out,
                            void* t_best_out, int32_t* trace, void* trace_t) {
    if (x0) DMMV_TRY(dmmv_set_x(c, x0));
    if (!c->x_set) return fail(DMMV_ERR_STATE, "dmmv_alns: no starting point (x0 is NULL and dmmv_set_x was never called)");
    DMMV_TRY(residual_any(c));
    if (c->p.n == 0) {
        DMMV_TRY(alns_start(c, false));
        DMMV_TRY(alns_export(c, t_best_out));
        DMMV_HIP_CHECK(hipStreamSynchronize(c->stream));
        return DMMV_OK;
    }
    int64_t count = prm.destroy_count > 0 ? prm.destroy_count : (c->p.n * 5 + 999) / 1000;
    if (count < 1) count = 1;
    if (count > c->p.n) count = c->p.n;
    // the local search runs with its own neighbourhood and always stops at a local optimum
    const dmmv_options saved = c->o;
    c->o.radius = prm.ls_radius;
    c->o.keep_going = 0;
    dmmv_status st = [&]() -> dmmv_status {
        DMMV_TRY(alns_start(c, prm.l2_guard != 0));
        for (int32_t it = 0; it < prm.iters; ++it) {
            DMMV_TRY(alns_destroy_repair(c, prm, it, (int32_t)count));
            if (batched_pruned_applicable(c)) {
                DMMV_TRY(batched_descent_pruned(c, prm.ls_moves, prm.ls_moves, nullptr, nullptr));
            } else {
                for (int32_t mv = 0; mv < prm.ls_moves; ++mv) DMMV_TRY(loop_step(c, prm.ls_moves, nullptr, nullptr));
            }
            if (prm.ls_swaps > 0) {
                DMMV_TRY(swap_clear_skip(c));
                for (int32_t sw = 0; sw < prm.ls_swaps; ++sw)
                    DMMV_TRY(swap_move(c, prm.k_eps, 1, true, nullptr, nullptr));
            }
            DMMV_TRY(alns_finish_iteration(c, prm, trace, trace_t));
        }
        DMMV_TRY(alns_export(c, t_best_out));
        return DMMV_OK;
    }();
    c->o = saved;
    DMMV_TRY(st);
    if (x_best_out && c->kind == KIND_BATCHED) {
        DMMV_TRY(batched_get_x_from(c, c->alns_kidx_best, x_best_out));
    } else if (x_best_out) {
        if (c->p.dtype == DMMV_F64)
            hipLaunchKernelGGL(k_index_to_values<double>, grid1(c->p.n, 256), dim3(256), 0, c->stream,
                               (const int32_t*)c->alns_kidx_best, (const double*)c->D_dev, c->p.n, (double*)x_best_out);
        else
            hipLaunchKernelGGL(k_index_to_values<float>, grid1(c->p.n, 256), dim3(256), 0, c->stream,
                               (const int32_t*)c->alns_kidx_best, (const float*)c->D_dev, c->p.n, (float*)x_best_out);
        DMMV_LAUNCH_CHECK();
    }
    DMMV_HIP_CHECK(hipStreamSynchronize(c->stream));
    return DMMV_OK;
}

// ----------------------------------------------------------------------------------------
// options and context set-up shared by dmmv_create and dmmv_solve_static
// ----------------------------------------------------------------------------------------
static dmmv_status resolve_options(const dmmv_problem* problem, const dmmv_options* options, dmmv_options* out) {
    DMMV_TRY(validate_problem(problem));
    dmmv_options o{};
    o.poll_every = 64;
    if (options) o = *options;
    if (o.radius < 0 || o.poll_every < 0 || o.sparse_partition_rows < 0)
        return fail(DMMV_ERR_SHAPE, "options: radius, poll_every and sparse_partition_rows must be >= 0");
    if (o.batched_eval < 0 || o.batched_eval > 2)
        return fail(DMMV_ERR_SHAPE, "options.batched_eval must be 0, 1 or 2");
    if (o.l2_rule < 0 || o.l2_rule > 3)
        return fail(DMMV_ERR_SHAPE, "options.l2_rule must be 0, 1, 2 or 3");
    if (o.sparse_eval < 0 || o.sparse_eval > 2)
        return fail(DMMV_ERR_SHAPE, "options.sparse_eval must be 0, 1 or 2");
    if (o.dense_loop < 0 || o.dense_loop > 2 || o.wait_limit < 0)
        return fail(DMMV_ERR_SHAPE, "options.dense_loop must be 0, 1 or 2 and wait_limit >= 0");
    if (o.dense_loop == 2 && !dense_persistent_fits(*problem))
        return fail(DMMV_ERR_UNSUPPORTED, "options.dense_loop = 2 needs one dense instance whose r, D, x and one column of A "
                    "fit 156 KiB of LDS");
    if (o.sparse_eval == 2 && problem->csr_rowptr) {
        int64_t mp, P;
        sparse_partitions(*problem, o, &mp, &P);
        if (P > 16) return fail(DMMV_ERR_UNSUPPORTED, "options.sparse_eval = 2 takes at most 16 row partitions (%lld here)", (long long)P);
    }
    if (problem->csr_rowptr) {
        // the partition count the layout will really use decides whether the matrix fits: every
        // (row partition, column) segment is padded to a multiple of four entries and holds at
        // least four, segment offsets are 32-bit, and the partitions are one grid dimension
        int64_t mp, P;
        sparse_partitions(*problem, o, &mp, &P);
        if (P > CSC_MAX_PARTITIONS)
            return fail(DMMV_ERR_UNSUPPORTED, "sparse path: %lld row partitions of %lld rows exceed the limit of %d (raise sparse_partition_rows)",
                        (long long)P, (long long)mp, CSC_MAX_PARTITIONS);
        if (problem->nnz + 4 * P * problem->n + 4 > (int64_t)INT32_MAX - 1)
            return fail(DMMV_ERR_UNSUPPORTED, "sparse matrix too large for 32-bit segment offsets (nnz + 4 * partitions * n must stay below 2^31)");
    }
    if (o.batched_eval == 2) {
        const bool is_batched = !problem->csr_rowptr && (problem->R > 1 || problem->scale);
        if (!is_batched || !batched_eval_mfma_applicable(*problem))
            return fail(DMMV_ERR_UNSUPPORTED, "options.batched_eval = 2 needs an fp32 batched problem with nd <= 32");
    }
    if (o.residual_mfma) {
        // the matrix-core residual needs fp32, the batched layout and codes that bf16 holds exactly
        const bool is_batched = !problem->csr_rowptr && (problem->R > 1 || problem->scale);
        if (problem->dtype != DMMV_F32 || !is_batched)
            return fail(DMMV_ERR_UNSUPPORTED, "options.residual_mfma needs an fp32 batched problem (R > 1 or scale given)");
        for (int32_t k = 0; k < problem->nd; ++k) {
            uint32_t bits;
            memcpy(&bits, (const float*)problem->D + k, sizeof(bits));
            if (bits & 0xFFFFu)
                return fail(DMMV_ERR_UNSUPPORTED, "options.residual_mfma: D[%d] is not exactly representable in bf16", k);
        }
    }
    *out = o;
    return DMMV_OK;
}

// Fill *c for a validated problem and build the internal layouts in `workspace` (large enough,
// 256-byte aligned).  Waits for the stream.
static dmmv_status ctx_setup(dmmv_ctx* c, const dmmv_problem* problem, const dmmv_options& o, void* workspace,
                             hipStream_t stream) {
    c->p = *problem;
    c->o = o;
    c->stream = stream;
    c->esz = problem->dtype == DMMV_F64 ? 8 : 4;
    const bool sparse = problem->csr_rowptr != nullptr;
    c->kind = sparse ? KIND_CSC : ((problem->R > 1 || problem->scale) ? KIND_BATCHED : KIND_DENSE);
    c->x_set = c->r_valid = false;
    c->cmp_on = false;
    workspace_layout(*problem, o, c, (char*)workspace);
    c->p.D = nullptr;       // host arrays are copied below and not referenced afterwards
    c->p.scale = nullptr;

    hipLaunchKernelGGL(k_zero_flags, dim3(1), dim3(64), 0, c->stream, c->flags);
    DMMV_HIP_CHECK(hipMemcpyAsync(c->D_dev, problem->D, (size_t)problem->nd * c->esz, hipMemcpyHostToDevice, c->stream));
    if (problem->scale) {
        DMMV_HIP_CHECK(hipMemcpyAsync(c->scale_dev, problem->scale, (size_t)problem->R * c->esz, hipMemcpyHostToDevice, c->stream));
    } else {
        static const double one_d = 1.0;     // static: the copy may read them after this block
        static const float one_f = 1.0f;
        const void* one = problem->dtype == DMMV_F64 ? (const void*)&one_d : (const void*)&one_f;
        DMMV_HIP_CHECK(hipMemcpyAsync(c->scale_dev, one, c->esz, hipMemcpyHostToDevice, c->stream));
    }
    // the host copies above read caller memory: they are finished before returning (the
    // stream is waited for below)
    if (problem->dtype == DMMV_F64)
        hipLaunchKernelGGL(k_init_state<double>, grid1(problem->R, 256), dim3(256), 0, c->stream, (InstState<double>*)c->state, problem->R);
    else
        hipLaunchKernelGGL(k_init_state<float>, grid1(problem->R, 256), dim3(256), 0, c->stream, (InstState<float>*)c->state, problem->R);
    DMMV_LAUNCH_CHECK();
    c->csc_max_row = 0;
    c->csc_max_col = 0;
    if (c->kind == KIND_CSC) {
        DMMV_TRY(csc_build(c));
        DMMV_HIP_CHECK(hipMemcpyAsync(&c->csc_max_row, &c->flags[FLAG_MAXROW], sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
        DMMV_HIP_CHECK(hipMemcpyAsync(&c->csc_max_col, &c->flags[FLAG_MAXCOL], sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
        DMMV_HIP_CHECK(hipStreamSynchronize(c->stream));
        if (c->csc_max_row > c->p.n) c->csc_max_row = (int32_t)c->p.n;   // duplicates are an error anyway
    }
    if (c->kind == KIND_BATCHED) DMMV_TRY(batched_build(c));
    if (c->kind == KIND_DENSE && o.prune) DMMV_TRY(batched_build_xt(c));
    if (o.l2_rule) DMMV_TRY(l2_build(c));
    c->mfma_planes = 1;
    if (o.residual_mfma) {
        DMMV_TRY(batched_mfma_build(c));
        int32_t lower = 0;
        DMMV_HIP_CHECK(hipMemcpyAsync(&lower, &c->flags[FLAG_PLANES], sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
        DMMV_HIP_CHECK(hipStreamSynchronize(c->stream));
        c->mfma_planes |= lower & 6;
    }
    return check_device_errors(c);
}

}  // namespace dmmv

// ========================================================================================
// C ABI
// ========================================================================================
using namespace dmmv;

extern "C" {

const char* dmmv_last_error(void) { return g_err; }
const char* dmmv_version(void) { return "libdmmv 0.1 (gfx950)"; }

size_t dmmv_workspace_bytes(const dmmv_problem* problem, const dmmv_options* options) {
    dmmv_options o{};
    if (resolve_options(problem, options, &o) != DMMV_OK) return 0;
    return workspace_layout(*problem, o, nullptr, nullptr);
}

dmmv_status dmmv_create(dmmv_handle* out, const dmmv_problem* problem, const dmmv_options* options,
                        void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!out) return fail(DMMV_ERR_NULL, "out handle pointer is NULL");
    *out = nullptr;
    dmmv_options o{};
    DMMV_TRY(resolve_options(problem, options, &o));
    const size_t need = workspace_layout(*problem, o, nullptr, nullptr);
    if (!workspace) return fail(DMMV_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", need);
    if (((uintptr_t)workspace & 255) != 0) return fail(DMMV_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    if (workspace_bytes < need) return fail(DMMV_ERR_WORKSPACE, "workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);

    dmmv_ctx* c = new (std::nothrow) dmmv_ctx();
    if (!c) return fail(DMMV_ERR_STATE, "out of host memory");
    const dmmv_status st = ctx_setup(c, problem, o, workspace, (hipStream_t)hip_stream);
    if (st != DMMV_OK) { delete c; return st; }
    *out = c;
    return DMMV_OK;
}

// ---- one-shot descent for callers that cannot allocate device memory ----------------------
// The workspace is an array in the library's own device image.  In host code the array's name is
// only a stand-in for the symbol: its device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[DMMV_STATIC_SCRATCH_BYTES];

namespace {
constexpr int SCRATCH_MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[SCRATCH_MAX_DEVICES] = {};

// device address of `scratch` on the current device
dmmv_status scratch_of_current_device(void** out) {
    int dev = -1;
    DMMV_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= SCRATCH_MAX_DEVICES) return fail(DMMV_ERR_UNSUPPORTED, "device ordinal %d outside [0, %d)", dev, SCRATCH_MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        DMMV_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || ((uintptr_t)ptr & 255) != 0) return fail(DMMV_ERR_HIP, "hipGetSymbolAddress gave an unusable address %p", ptr);
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return DMMV_OK;
}
}  // namespace

dmmv_status dmmv_solve_static(const dmmv_problem* problem, const dmmv_options* options, const void* x0,
                              int32_t iters, void* x_out, void* max_violation_out, int32_t* iters_done,
                              dmmv_move* trace, void* trace_t, void* hip_stream) {
    if (iters < 0) return fail(DMMV_ERR_SHAPE, "iters must be >= 0");
    dmmv_options o{};
    DMMV_TRY(resolve_options(problem, options, &o));
    if (!x0 && problem->n > 0) return fail(DMMV_ERR_NULL, "dmmv_solve_static: x0 is NULL");
    const size_t need = workspace_layout(*problem, o, nullptr, nullptr);
    if (need > (size_t)DMMV_STATIC_SCRATCH_BYTES)
        return fail(DMMV_ERR_WORKSPACE, "dmmv_solve_static: this problem needs %zu bytes of workspace, the built-in scratch holds %zu "
                    "(use dmmv_create with a workspace of your own)", need, (size_t)DMMV_STATIC_SCRATCH_BYTES);
    void* ws = nullptr;
    DMMV_TRY(scratch_of_current_device(&ws));
    dmmv_ctx c{};                                          // on the stack: nothing is allocated
    DMMV_TRY(ctx_setup(&c, problem, o, ws, (hipStream_t)hip_stream));
    const dmmv_status st = dmmv_solve(&c, x0, iters, x_out, max_violation_out, iters_done, trace, trace_t);
    if (st != DMMV_OK) (void)hipStreamSynchronize(c.stream);   // nothing of this call may still use the scratch
    return st;
}

dmmv_status dmmv_destroy(dmmv_handle h) {
    if (!h) return fail(DMMV_ERR_NULL, "handle is NULL");
    (void)hipStreamSynchronize(h->stream);
    delete h;
    return DMMV_OK;
}

dmmv_status dmmv_set_x(dmmv_handle h, const void* x_values) {
    if (!h) return fail(DMMV_ERR_NULL, "handle is NULL");
    if (!x_values && h->p.n > 0) return fail(DMMV_ERR_NULL, "x_values is NULL");
    h->x_set = false;
    h->r_valid = false;
    if (h->p.n > 0) {
        if (h->kind == KIND_BATCHED) DMMV_TRY(batched_set_x(h, x_values));
        else if (h->p.dtype == DMMV_F64) DMMV_TRY(set_x_single<double>(h, x_values));
        else DMMV_TRY(set_x_single<float>(h, x_values));
    }
    DMMV_TRY(check_device_errors(h));
    h->x_set = true;
    return DMMV_OK;
}

dmmv_status dmmv_set_residual(dmmv_handle h, const void* r) {
    if (!h) return fail(DMMV_ERR_NULL, "handle is NULL");
    if (!r && h->p.m > 0) return fail(DMMV_ERR_NULL, "r is NULL");
    if (!h->x_set) return fail(DMMV_ERR_STATE, "dmmv_set_residual before dmmv_set_x");
    if (h->p.m > 0) {
        if (h->kind == KIND_BATCHED) DMMV_TRY(batched_set_r(h, r));
        else DMMV_HIP_CHECK(hipMemcpyAsync(h->r, r, (size_t)h->p.m * h->esz, hipMemcpyDeviceToDevice, h->stream));
    }
    DMMV_TRY(refresh_t(h));
    h->r_valid = true;
    return DMMV_OK;
}

dmmv_status dmmv_residual(dmmv_handle h, void* r_out) {
    if (!h) return fail(DMMV_ERR_NULL, "handle is NULL");
    if (!h->x_set) return fail(DMMV_ERR_STATE, "dmmv_residual before dmmv_set_x");
    DMMV_TRY(residual_any(h));
    if (r_out) DMMV_TRY(dmmv_get_state(h, nullptr, r_out, nullptr));
    return DMMV_OK;
}

dmmv_status dmmv_eval_moves(dmmv_handle h, void* scores_out) {
    if (!h) return fail(DMMV_ERR_NULL, "handle is NULL");
    if (!scores_out && h->p.n > 0) return fail(DMMV_ERR_NULL, "scores_out is NULL");
    if (!h->r_valid) return fail(DMMV_ERR_STATE, "dmmv_eval_moves needs a residual (call dmmv_residual or dmmv_set_residual)");
    return eval_any(h, scores_out, false, false);
}

dmmv_status dmmv_argmin_move(dmmv_handle h, const void* scores, dmmv_move* best, void* best_score) {
    if (!h) return fail(DMMV_ERR_NULL, "handle is NULL");
    if (!best && !best_score) return fail(DMMV_ERR_NULL, "best and best_score are both NULL");
    const bool l2_on = h->o.l2_rule == 1 || h->o.l2_rule == 2;
    if (l2_on) {
        // the second criterion is a function of the current residual: the table given (or the
        // evaluation made here) is reduced together with the l2 changes of the current state
        if (!h->r_valid) return fail(DMMV_ERR_STATE, "dmmv_argmin_move with options.l2_rule needs a residual");
        if (h->p.n == 0) {
            if (best) DMMV_HIP_CHECK(hipMemsetAsync(best, 0xFF, (size_t)h->p.R * sizeof(dmmv_move), h->stream));
            return DMMV_OK;
        }
        if (h->p.dtype == DMMV_F64)
            hipLaunchKernelGGL(k_clear_done<double>, grid1(h->p.R, 256), dim3(256), 0, h->stream, (InstState<double>*)h->state, h->p.R);
        else
            hipLaunchKernelGGL(k_clear_done<float>, grid1(h->p.R, 256), dim3(256), 0, h->stream, (InstState<float>*)h->state, h->p.R);
        if (!scores) DMMV_TRY(eval_any(h, h->l2_scores, false, false));
        DMMV_TRY(l2_update_g(h));
        return l2_select(h, scores ? scores : h->l2_scores, 1, best, best_score);
    }
    if (scores) {
        const int64_t ntab = h->p.n * (int64_t)h->p.nd;
        if (h->p.dtype == DMMV_F64)
            hipLaunchKernelGGL(k_argmin_table<double>, dim3((unsigned)h->p.R), dim3(1024), 0, h->stream, (const double*)scores, ntab, h->p.nd, best, (double*)best_score);
        else
            hipLaunchKernelGGL(k_argmin_table<float>, dim3((unsigned)h->p.R), dim3(1024), 0, h->stream, (const float*)scores, ntab, h->p.nd, best, (float*)best_score);
        DMMV_LAUNCH_CHECK();
        return DMMV_OK;
    }
    if (!h->r_valid) return fail(DMMV_ERR_STATE, "dmmv_argmin_move(scores = NULL) needs a residual");
    const int32_t keep = h->o.keep_going;
    h->o.keep_going = 1;   // a standalone query must not stop the instance
    if (h->p.dtype == DMMV_F64)
        hipLaunchKernelGGL(k_clear_done<double>, grid1(h->p.R, 256), dim3(256), 0, h->stream, (InstState<double>*)h->state, h->p.R);
    else
        hipLaunchKernelGGL(k_clear_done<float>, grid1(h->p.R, 256), dim3(256), 0, h->stream, (InstState<float>*)h->state, h->p.R);
    dmmv_status st = eval_any(h, nullptr, true, false);
    if (st == DMMV_OK) st = launch_select(h, best, best_score);
    h->o.keep_going = keep;
    return st;
}

dmmv_status dmmv_apply_move(dmmv_handle h, const dmmv_move* moves) {
    if (!h) return fail(DMMV_ERR_NULL, "handle is NULL");
    if (!moves) return fail(DMMV_ERR_NULL, "moves is NULL");
    if (!h->r_valid) return fail(DMMV_ERR_STATE, "dmmv_apply_move needs a residual");
    const int64_t R = h->p.R;
    const bool batched = h->kind == KIND_BATCHED;
    if (h->p.dtype == DMMV_F64)
        hipLaunchKernelGGL(k_stage_moves<double>, grid1(R, 256), dim3(256), 0, h->stream, moves, R, h->p.n, h->p.nd, (InstState<double>*)h->state, (const double*)h->D_dev, batched ? (const double*)h->scale_dev : nullptr, (const int32_t*)h->kidx, h->flags);
    else
        hipLaunchKernelGGL(k_stage_moves<float>, grid1(R, 256), dim3(256), 0, h->stream, moves, R, h->p.n, h->p.nd, (InstState<float>*)h->state, (const float*)h->D_dev, batched ? (const float*)h->scale_dev : nullptr, (const int32_t*)h->kidx, h->flags);
    DMMV_LAUNCH_CHECK();
    DMMV_TRY(check_device_errors(h));
    DMMV_TRY(apply_any(h, false, 0, nullptr, nullptr));
    DMMV_TRY(refresh_t(h));
    return DMMV_OK;
}

dmmv_status dmmv_get_state(dmmv_handle h, void* x_values, void* r, void* max_violation) {
    if (!h) return fail(DMMV_ERR_NULL, "handle is NULL");
    const int64_t R = h->p.R;
    if (x_values && h->p.n > 0) {
        if (!h->x_set) return fail(DMMV_ERR_STATE, "dmmv_get_state: x was never set");
        if (h->kind == KIND_BATCHED) DMMV_TRY(batched_get_x(h, x_values));
        else if (h->p.dtype == DMMV_F64)
            hipLaunchKernelGGL(k_index_to_values<double>, grid1(h->p.n, 256), dim3(256), 0, h->stream, (const int32_t*)h->kidx, (const double*)h->D_dev, h->p.n, (double*)x_values);
        else
            hipLaunchKernelGGL(k_index_to_values<float>, grid1(h->p.n, 256), dim3(256), 0, h->stream, (const int32_t*)h->kidx, (const float*)h->D_dev, h->p.n, (float*)x_values);
    }
    if (r && h->p.m > 0) {
        if (!h->r_valid) return fail(DMMV_ERR_STATE, "dmmv_get_state: no residual yet");
        if (h->kind == KIND_BATCHED) DMMV_TRY(batched_get_r(h, r));
        else DMMV_HIP_CHECK(hipMemcpyAsync(r, h->r, (size_t)h->p.m * h->esz, hipMemcpyDeviceToDevice, h->stream));
    }
    if (max_violation) {
        if (!h->r_valid) return fail(DMMV_ERR_STATE, "dmmv_get_state: no residual yet");
        if (h->p.dtype == DMMV_F64)
            hipLaunchKernelGGL(k_export_state<double>, grid1(R, 256), dim3(256), 0, h->stream, (const InstState<double>*)h->state, R, (double*)max_violation, (int32_t*)nullptr);
        else
            hipLaunchKernelGGL(k_export_state<float>, grid1(R, 256), dim3(256), 0, h->stream, (const InstState<float>*)h->state, R, (float*)max_violation, (int32_t*)nullptr);
    }
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

dmmv_status dmmv_solve(dmmv_handle h, const void* x0, int32_t iters, void* x_out,
                       void* max_violation_out, int32_t* iters_done, dmmv_move* trace,
                       void* trace_t) {
    if (!h) return fail(DMMV_ERR_NULL, "handle is NULL");
    if (iters < 0) return fail(DMMV_ERR_SHAPE, "iters must be >= 0");
    return h->p.dtype == DMMV_F64
               ? solve_t<double>(h, x0, iters, x_out, max_violation_out, iters_done, trace, trace_t)
               : solve_t<float>(h, x0, iters, x_out, max_violation_out, iters_done, trace, trace_t);
}

dmmv_status dmmv_alns(dmmv_handle h, const void* x0, const dmmv_alns_params* params, void* x_best_out,
                      void* t_best_out, int32_t* trace, void* trace_t) {
    if (!h) return fail(DMMV_ERR_NULL, "handle is NULL");
    if (!params) return fail(DMMV_ERR_NULL, "params is NULL");
    if (h->kind == KIND_BATCHED && !h->o.alns)
        return fail(DMMV_ERR_STATE, "dmmv_alns: a batched handle needs options.alns = 1 at dmmv_create (workspace for the outer loop)");
    if (params->iters < 0 || params->ls_moves < 0 || params->ls_radius < 0 || params->destroy_count < 0)
        return fail(DMMV_ERR_SHAPE, "dmmv_alns: iters, ls_moves, ls_radius and destroy_count must be >= 0");
    if (params->ls_swaps < 0 || params->k_eps < 0)
        return fail(DMMV_ERR_SHAPE, "dmmv_alns: ls_swaps and k_eps must be >= 0");
    if ((params->l2_guard != 0 && params->l2_guard != 1) || params->reserved != 0)
        return fail(DMMV_ERR_DOMAIN, "dmmv_alns: l2_guard must be 0 or 1 and reserved 0");
    if (!(params->alpha >= 0.0) || !(params->lambda >= 0.0 && params->lambda <= 1.0) ||
        !(params->sigma1 >= 0.0) || !(params->sigma2 >= 0.0) || !(params->sigma3 >= 0.0))
        return fail(DMMV_ERR_DOMAIN, "dmmv_alns: need alpha >= 0, 0 <= lambda <= 1, sigma >= 0");
    return alns_run(h, x0, *params, x_best_out, t_best_out, trace, trace_t);
}

dmmv_status dmmv_l2_changes(dmmv_handle h, void* dq_out) {
    if (!h) return fail(DMMV_ERR_NULL, "handle is NULL");
    if (!dq_out && h->p.n > 0) return fail(DMMV_ERR_NULL, "dq_out is NULL");
    if (!h->o.l2_rule) return fail(DMMV_ERR_STATE, "dmmv_l2_changes needs a handle created with options.l2_rule != 0 (workspace for g and the column norms)");
    if (!h->r_valid) return fail(DMMV_ERR_STATE, "dmmv_l2_changes needs a residual (call dmmv_residual or dmmv_set_residual)");
    DMMV_TRY(l2_update_g(h));
    return l2_table(h, dq_out);
}

dmmv_status dmmv_swap_move(dmmv_handle h, int32_t k_eps, int32_t apply, dmmv_swap* best, void* best_t) {
    if (!h) return fail(DMMV_ERR_NULL, "dmmv_swap_move: handle is NULL");
    if (k_eps < 0) return fail(DMMV_ERR_SHAPE, "dmmv_swap_move: k_eps < 0");
    if (!h->r_valid) return fail(DMMV_ERR_STATE, "dmmv_swap_move: no residual (call dmmv_residual or dmmv_solve first)");
    return swap_move(h, k_eps, apply, false, best, best_t);
}

int32_t dmmv_loop_in_use(dmmv_handle h) {
    if (!h) return 0;
    return (batched_pruned_applicable(h) || dense_persistent_applicable(h)) ? 2 : 1;
}

dmmv_status dmmv_time_eval(dmmv_handle h, int32_t reps, float* ms_out) {
    if (!h) return fail(DMMV_ERR_NULL, "handle is NULL");
    if (!ms_out) return fail(DMMV_ERR_NULL, "ms_out is NULL");
    if (reps == 0) return fail(DMMV_ERR_SHAPE, "reps must not be 0");
    const bool warm = reps > 0;
    if (!warm) reps = -reps;
    if (!h->r_valid) return fail(DMMV_ERR_STATE, "dmmv_time_eval needs a residual");
    if (h->p.dtype == DMMV_F64)
        hipLaunchKernelGGL(k_clear_done<double>, grid1(h->p.R, 256), dim3(256), 0, h->stream, (InstState<double>*)h->state, h->p.R);
    else
        hipLaunchKernelGGL(k_clear_done<float>, grid1(h->p.R, 256), dim3(256), 0, h->stream, (InstState<float>*)h->state, h->p.R);
    hipEvent_t e0, e1;
    DMMV_HIP_CHECK(hipEventCreate(&e0));
    DMMV_HIP_CHECK(hipEventCreate(&e1));
    // the whole evaluation step as the descent runs it (sparse, two-kernel path: both kernels)
    auto once = [&]() { return eval_any(h, nullptr, true, false); };
    dmmv_status st = (warm && h->p.n > 0) ? once() : DMMV_OK;       // warm-up launch, not timed
    if (st == DMMV_OK) {
        (void)hipEventRecord(e0, h->stream);
        for (int32_t q = 0; q < reps && st == DMMV_OK && h->p.n > 0; ++q) st = once();
        (void)hipEventRecord(e1, h->stream);
        hipError_t e = hipEventSynchronize(e1);
        if (e != hipSuccess) st = fail(DMMV_ERR_HIP, "hipEventSynchronize failed: %s", hipGetErrorString(e));
        else (void)hipEventElapsedTime(ms_out, e0, e1);
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return st;
}

dmmv_status dmmv_time_l2(dmmv_handle h, int32_t reps, float* ms_out) {
    if (!h) return fail(DMMV_ERR_NULL, "handle is NULL");
    if (!ms_out) return fail(DMMV_ERR_NULL, "ms_out is NULL");
    if (reps < 1) return fail(DMMV_ERR_SHAPE, "reps must be >= 1");
    if (!h->o.l2_rule) return fail(DMMV_ERR_STATE, "dmmv_time_l2 needs a handle created with options.l2_rule != 0");
    if (!h->r_valid) return fail(DMMV_ERR_STATE, "dmmv_time_l2 needs a residual");
    hipEvent_t e0, e1;
    DMMV_HIP_CHECK(hipEventCreate(&e0));
    DMMV_HIP_CHECK(hipEventCreate(&e1));
    dmmv_status st = l2_update_g(h);                       // warm-up launch, not timed
    if (st == DMMV_OK) {
        (void)hipEventRecord(e0, h->stream);
        for (int32_t q = 0; q < reps && st == DMMV_OK; ++q) st = l2_update_g(h);
        (void)hipEventRecord(e1, h->stream);
        hipError_t e = hipEventSynchronize(e1);
        if (e != hipSuccess) st = fail(DMMV_ERR_HIP, "hipEventSynchronize failed: %s", hipGetErrorString(e));
        else (void)hipEventElapsedTime(ms_out, e0, e1);
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return st;
}

}  // extern "C"
