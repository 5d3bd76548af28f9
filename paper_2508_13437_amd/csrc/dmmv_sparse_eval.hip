// Sparse move evaluation: a streaming kernel and a finalize kernel.
//
// k_eval_stream.  grid = (workgroups per partition, partitions).  A workgroup stages ITS
// partition of r in LDS once (64 KiB, so two workgroups share a compute unit: one stages while
// the other streams) and owns a range of columns holding an equal share of the partition's
// entries.  ST_LPC adjacent lanes take one column segment, 64 entries per pass: each lane
// loads aligned groups of four consecutive entries (one 8-byte load of row offsets, one
// 16-byte load of values, coalesced and unconditional: a lane past its segment re-reads the
// segment's last group), gathers r from LDS, keeps KT running maxima and reduces them over
// the column's lanes with integer DPP max.  Every wavefront keeps DEPTH column groups in
// flight: the loads of group g + DEPTH*8 go out right after group g is consumed.
// Output: per partition, the maximum over the touched rows for every (column, value), and
// the mask of the first RES_FAST reservoir rows the column meets in this partition.
//
// k_finalize_csc.  One thread per column: combine the partitions, add the maximum over the
// rows OUTSIDE the column (first reservoir row the column does not contain; rare columns that
// contain every inline-checked row walk the rest of the reservoir, then scan all rows),
// apply the neighbourhood mask, write scores and one arg-min record per workgroup.
#include <type_traits>

#include "dmmv_sparse_common.h"

namespace dmmv {

constexpr int ST_BLOCK = 512;
constexpr int ST_WAVES = ST_BLOCK / 64;
constexpr int ST_LPC = 8;          // lanes that share a column (4, 8 or 16)
constexpr int ST_QPL = 16 / ST_LPC;    // aligned groups of four entries per lane per pass (64 entries per column)
constexpr int ST_CPW = 64 / ST_LPC;    // columns a wavefront works on at a time
constexpr int ST_DEPTH = 4 / ST_QPL > 1 ? 4 / ST_QPL : 2;   // column groups a wavefront keeps in flight
constexpr int ST_COLS = 1024;      // columns whose bounds / current values sit in LDS at once
constexpr int FIN_BLOCK = CSC_FIN_BLOCK;

// one pass (64 entries per column) of one group of ST_CPW columns, as loaded: per lane ST_QPL
// groups of four consecutive entries, 4 * ST_LPC entries apart
template <class T>
struct EntryRegs {
    uint2 ix[ST_QPL];
    typename Vec4<T>::type av[ST_QPL];
};

// Every segment holds at least one aligned group of four entries (pads included), so a lane
// whose entries would lie past its segment reads the segment's last group again instead: a
// repeated entry changes neither a maximum nor a mask, and no lane needs masking.
template <class T>
__device__ __forceinline__ void load_entries(EntryRegs<T>& E, const uint16_t* __restrict__ row16,
                                             const T* __restrict__ cval, int32_t e, int32_t s1) {
#pragma unroll
    for (int g = 0; g < ST_QPL; ++g) {
        const int32_t eg = e + g * (SEG_ALIGN * ST_LPC);
        const int32_t ec = eg < s1 ? eg : s1 - SEG_ALIGN;
        E.ix[g] = *reinterpret_cast<const uint2*>(row16 + ec);
        E.av[g] = *reinterpret_cast<const typename Vec4<T>::type*>(cval + ec);
    }
}

// fold one pass into the lane's running maxima and reservoir mask
template <class T, int KT>
__device__ __forceinline__ void fold_pass(const EntryRegs<T>& E, const T* lds_r, const T (&delta)[KT],
                                          T (&acc)[KT], uint32_t& mask, bool first_tile, T thr,
                                          int32_t nfast, const int32_t* sh_rloc) {
#pragma unroll
    for (int g = 0; g < ST_QPL; ++g) {
        const uint32_t i0 = E.ix[g].x & 0xFFFFu, i1 = E.ix[g].x >> 16, i2 = E.ix[g].y & 0xFFFFu, i3 = E.ix[g].y >> 16;
        const T r0 = lds_r[i0], r1 = lds_r[i1], r2 = lds_r[i2], r3 = lds_r[i3];
        if (first_tile) {
            const T big = dmmv_max(dmmv_max(dmmv_abs(r0), dmmv_abs(r1)), dmmv_max(dmmv_abs(r2), dmmv_abs(r3)));
            if (big >= thr) {      // uncommon: one of these rows may be among the listed ones
                for (int32_t q = 0; q < nfast; ++q) {
                    const uint32_t l = (uint32_t)sh_rloc[q];     // offset in this partition or ~0
                    if (i0 == l || i1 == l || i2 == l || i3 == l) mask |= 1u << q;
                }
            }
        }
#pragma unroll
        for (int q = 0; q < KT; ++q) {
            T a = acc[q];
            a = dmmv_max(a, dmmv_abs(dmmv_fma(delta[q], E.av[g].x, r0)));
            a = dmmv_max(a, dmmv_abs(dmmv_fma(delta[q], E.av[g].y, r1)));
            a = dmmv_max(a, dmmv_abs(dmmv_fma(delta[q], E.av[g].z, r2)));
            a = dmmv_max(a, dmmv_abs(dmmv_fma(delta[q], E.av[g].w, r3)));
            acc[q] = a;
        }
    }
}

template <class T, int KT>
__global__ __launch_bounds__(ST_BLOCK, 4) void k_eval_stream(   // 4 waves per SIMD: 2 workgroups per CU
    int64_t m, int64_t n, int32_t nd, int32_t mp, const int32_t* __restrict__ segptr,
    const uint16_t* __restrict__ row16, const T* __restrict__ cval,
    const int32_t* __restrict__ blk_lo, const T* __restrict__ D, const int32_t* __restrict__ kidx,
    const T* __restrict__ r, const T* __restrict__ res_val, const int32_t* __restrict__ res_row,
    const int32_t* __restrict__ res_meta, const InstState<T>* __restrict__ st, int32_t honor_done,
    T* __restrict__ part_scores, uint32_t* __restrict__ part_mask) {
    extern __shared__ __align__(32) unsigned char smem[];
    T* lds_r = reinterpret_cast<T*>(smem);                 // mp + 1 entries (slot mp = 0)
    __shared__ int32_t sh_b[ST_COLS + 1];
    __shared__ T sh_dcur[ST_COLS];
    __shared__ int32_t sh_rloc[RES_FAST];
    if (honor_done && st[0].done) return;

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int sub = lane & (ST_LPC - 1);       // position among the lanes of one column
    const int rowid = lane / ST_LPC;           // which of the wavefront's columns
    const int32_t p = blockIdx.y;
    const int64_t j_lo = blk_lo[p * (gridDim.x + 1) + blockIdx.x];
    const int64_t j_hi = blk_lo[p * (gridDim.x + 1) + blockIdx.x + 1];
    const int64_t row0 = (int64_t)p * mp;
    const int32_t rows_here = (int32_t)((m - row0) < mp ? (m - row0) : mp);
    const int32_t cnt = res_meta[RES_CNT];
    const int32_t nfast = cnt < RES_FAST ? cnt : RES_FAST;
    const T thr = nfast > 0 ? res_val[nfast - 1] : Limits<T>::inf();
    if (threadIdx.x < RES_FAST) {
        // offset of the q-th reservoir row inside this partition (no such offset otherwise)
        int32_t loc = -1;
        if ((int32_t)threadIdx.x < nfast) {
            const int64_t d = (int64_t)res_row[threadIdx.x] - row0;
            if (d >= 0 && d < (int64_t)rows_here) loc = (int32_t)d;
        }
        sh_rloc[threadIdx.x] = loc;
    }
    bool r_staged = false;

    const int32_t* __restrict__ sp = segptr + (int64_t)p * n;
    T* __restrict__ out = part_scores + (int64_t)p * (n * (int64_t)nd);
    uint32_t* __restrict__ out_mask = part_mask + (int64_t)p * n;

    for (int64_t c0 = j_lo; c0 < j_hi; c0 += ST_COLS) {
        const int32_t nc = (int32_t)(j_hi - c0 < ST_COLS ? j_hi - c0 : ST_COLS);
        const int32_t nq = (nc + ST_CPW - 1) / ST_CPW;
        __syncthreads();                       // previous chunk consumed
        for (int32_t t = threadIdx.x; t <= nc; t += ST_BLOCK) {
            sh_b[t] = sp[c0 + t];
            if (t < nc) sh_dcur[t] = D[kidx[c0 + t]];
        }
        __syncthreads();                       // bounds and current values staged

        for (int32_t k0 = 0; k0 < nd; k0 += KT) {
            T dk[KT];
#pragma unroll
            for (int q = 0; q < KT; ++q) dk[q] = D[k0 + q < nd ? k0 + q : nd - 1];
            EntryRegs<T> ent[ST_DEPTH];
            int32_t qe[ST_DEPTH], qs1[ST_DEPTH];
#pragma unroll
            for (int u = 0; u < ST_DEPTH; ++u) {
                const int32_t t = (w + u * ST_WAVES) * ST_CPW + rowid;
                const bool okc = t < nc;
                qe[u] = (okc ? sh_b[t] : 0) + sub * SEG_ALIGN;
                qs1[u] = okc ? sh_b[t + 1] : SEG_ALIGN;        // no column: entries 0..3, unused
                load_entries<T>(ent[u], row16, cval, qe[u], qs1[u]);
            }
            if (!r_staged) {
                // stage this partition of r while the first groups' entries are in flight
                if ((row0 & 3) == 0) {
                    const int32_t nvec = rows_here >> 2;
                    const typename Vec4<T>::type* __restrict__ src = reinterpret_cast<const typename Vec4<T>::type*>(r + row0);
                    typename Vec4<T>::type* dst = reinterpret_cast<typename Vec4<T>::type*>(lds_r);
                    for (int32_t i = threadIdx.x; i < nvec; i += ST_BLOCK) dst[i] = src[i];
                    for (int32_t i = (nvec << 2) + threadIdx.x; i < rows_here; i += ST_BLOCK) lds_r[i] = r[row0 + i];
                } else {
                    for (int32_t i = threadIdx.x; i < rows_here; i += ST_BLOCK) lds_r[i] = r[row0 + i];
                }
                if (threadIdx.x == 0) lds_r[mp] = (T)0;
                r_staged = true;
                __syncthreads();
            }
            for (int32_t g0 = w; g0 < nq; g0 += ST_WAVES * ST_DEPTH) {
#pragma unroll
                for (int u = 0; u < ST_DEPTH; ++u) {
                    const int32_t g = g0 + u * ST_WAVES;
                    if (g < nq) {                              // uniform per wavefront
                        const int32_t t = g * ST_CPW + rowid;
                        const bool col_ok = t < nc;
                        const T dcur = sh_dcur[col_ok ? t : 0];
                        T delta[KT], acc[KT];
#pragma unroll
                        for (int q = 0; q < KT; ++q) { delta[q] = step_of(dk[q], dcur, (T)1); acc[q] = (T)0; }
                        uint32_t mask = 0;
                        fold_pass<T, KT>(ent[u], lds_r, delta, acc, mask, k0 == 0, thr, nfast, sh_rloc);
                        // segments longer than one pass (the columns of a wavefront diverge here)
                        const int32_t seg_end = qs1[u];
                        for (int32_t e = qe[u] + 64; e - sub * SEG_ALIGN < seg_end; e += 64) {
                            EntryRegs<T> more;
                            load_entries<T>(more, row16, cval, e, seg_end);
                            fold_pass<T, KT>(more, lds_r, delta, acc, mask, k0 == 0, thr, nfast, sh_rloc);
                        }
#pragma unroll
                        for (int q = 0; q < KT; ++q) acc[q] = lanes_max_nonneg<ST_LPC>(acc[q]);
                        if (k0 == 0) mask = lanes_or<ST_LPC>(mask);
                        if (sub == 0 && col_ok) {
                            const int64_t j = c0 + t;
#pragma unroll
                            for (int q = 0; q < KT; ++q)
                                if (k0 + q < nd) out[j * (int64_t)nd + k0 + q] = acc[q];
                            if (k0 == 0) out_mask[j] = mask;
                        }
                    }
                    // the group DEPTH * ST_WAVES further on takes this slot
                    {
                        const int32_t t = (g + ST_WAVES * ST_DEPTH) * ST_CPW + rowid;
                        const bool okc = t < nc;
                        qe[u] = (okc ? sh_b[t] : 0) + sub * SEG_ALIGN;
                        qs1[u] = okc ? sh_b[t + 1] : SEG_ALIGN;
                        load_entries<T>(ent[u], row16, cval, qe[u], qs1[u]);
                    }
                }
            }
        }
    }
}

// =========================================================================================
// one-kernel evaluation: every partition inside one workgroup
// =========================================================================================
// For matrices whose residual is a few partitions long, cutting the work by (partition, column
// range) costs a second kernel that only combines the partitions.  Here a workgroup of sixteen
// wavefronts owns FZ_COLS = 256 columns (two groups of eight per wavefront, eight lanes per
// column as above) and walks the partitions itself: the running maxima of its columns stay in
// registers from the first partition to the last.  The kernel lives on memory latency, so
// everything is requested early and nothing is spilled (a reload from scratch memory would queue
// behind every load in flight): the entries of a group for partition p + 1 are requested the
// moment its registers for partition p are folded, partition p + 1 of r travels from memory to
// the second LDS buffer (through registers) while the lanes fold partition p, and nothing waits
// at the barrier between two partitions but the barrier itself.  A lane takes two aligned groups
// of four entries of its column per partition (64 entries per column).  A group of eight columns
// with a segment longer than that (one in fourteen for the projection matrices this is written
// for) gets a third group of four per lane from a spare set of registers of the wavefront; what
// is longer still, or finds the spare set taken, goes on with loads that are waited for.  After
// the last partition the lanes add the maximum over the rows outside their column, apply the
// neighbourhood and reduce to ONE arg-min record per workgroup: no per-partition maxima leave
// the chip.  Every workgroup reads all of r (256 columns share one copy), which is why this
// kernel serves matrices with (n / 256) m w bytes of residual traffic not above the matrix
// itself; the two-kernel path serves the others.
constexpr int FZ_BLOCK = 1024;
constexpr int FZ_WAVES = FZ_BLOCK / 64;
constexpr int FZ_GROUPS = 2;                               // column groups per wavefront
constexpr int FZ_COLS = FZ_WAVES * ST_CPW * FZ_GROUPS;
constexpr int FZ_NQ = 2;                                   // aligned groups of four entries per lane per partition
constexpr int FZ_QSTEP = SEG_ALIGN * ST_LPC;               // entries of a column one such group covers over its lanes (32)
constexpr int FZ_RV = CSC_LDS_BYTES / 16 / FZ_BLOCK;       // 16-byte pieces of a partition of r per thread
constexpr int FZ_MAX_P = 16;                               // partitions whose segment bounds fit the LDS table
typedef uint32_t fz_piece __attribute__((ext_vector_type(4)));   // one such piece, a plain vector of registers
static_assert(FZ_COLS == CSC_FIN_BLOCK, "one arg-min record per 256 columns, as the two-kernel path writes");

// one aligned group of four entries: the lane's own, or the segment's last group when the lane's
// would lie past the segment (a repeated entry changes neither a maximum nor a mask)
template <class T>
__device__ __forceinline__ void fz_load_quad(uint2& ix, typename Vec4<T>::type& av,
                                             const uint16_t* __restrict__ row16, const T* __restrict__ cval,
                                             int32_t eg, int32_t s1) {
    const int32_t ec = eg < s1 ? eg : s1 - SEG_ALIGN;
    ix = *reinterpret_cast<const uint2*>(row16 + ec);
    av = *reinterpret_cast<const typename Vec4<T>::type*>(cval + ec);
}

// dk[q] - dcur is the step of value q (the unscaled instance: the factor 1 of step_of is exact)
template <class T, int KT>
__device__ __forceinline__ void fz_fold_quad(const uint2 ix, const typename Vec4<T>::type av, const T* lds_r,
                                             const T (&dk)[KT], T dcur, T (&acc)[KT], uint32_t& mask, bool first_tile,
                                             T thr, int32_t nfast, const int32_t* sh_rr, int64_t row0,
                                             int32_t rows_here) {
    const uint32_t i0 = ix.x & 0xFFFFu, i1 = ix.x >> 16, i2 = ix.y & 0xFFFFu, i3 = ix.y >> 16;
    const T r0 = lds_r[i0], r1 = lds_r[i1], r2 = lds_r[i2], r3 = lds_r[i3];
    if (first_tile) {
        const T big = dmmv_max(dmmv_max(dmmv_abs(r0), dmmv_abs(r1)), dmmv_max(dmmv_abs(r2), dmmv_abs(r3)));
        if (big >= thr) {      // uncommon: one of these rows may be among the listed ones
            for (int32_t q = 0; q < nfast; ++q) {
                const int64_t d = (int64_t)sh_rr[q] - row0;
                const uint32_t l = (d >= 0 && d < (int64_t)rows_here) ? (uint32_t)d : ~0u;
                if (i0 == l || i1 == l || i2 == l || i3 == l) mask |= 1u << q;
            }
        }
    }
#pragma unroll
    for (int q = 0; q < KT; ++q) {
        const T delta = step_of(dk[q], dcur, (T)1);
        T a = acc[q];
        a = dmmv_max(a, dmmv_abs(dmmv_fma(delta, av.x, r0)));
        a = dmmv_max(a, dmmv_abs(dmmv_fma(delta, av.y, r1)));
        a = dmmv_max(a, dmmv_abs(dmmv_fma(delta, av.z, r2)));
        a = dmmv_max(a, dmmv_abs(dmmv_fma(delta, av.w, r3)));
        acc[q] = a;
    }
}

template <class T, int KT>
__global__ __launch_bounds__(FZ_BLOCK) void k_eval_fused(
    int64_t m, int32_t n, int32_t nd, int32_t mp, int32_t P, const int32_t* __restrict__ segptr,
    const uint16_t* __restrict__ row16, const T* __restrict__ cval, const T* __restrict__ D,
    const int32_t* __restrict__ kidx, const T* __restrict__ r, const T* __restrict__ res_val,
    const int32_t* __restrict__ res_row, const int32_t* __restrict__ res_meta,
    const InstState<T>* __restrict__ st, int32_t honor_done, int32_t radius,
    const uint8_t* __restrict__ var_mask, T* __restrict__ scores, Partial<T>* __restrict__ part) {
    extern __shared__ __align__(32) unsigned char smem[];
    const int32_t buf_bytes = (int32_t)((((size_t)mp + 1) * sizeof(T) + 15) / 16 * 16);
    T* const buf0 = reinterpret_cast<T*>(smem);
    T* const buf1 = reinterpret_cast<T*>(smem + buf_bytes);
    int32_t* const sh_seg = reinterpret_cast<int32_t*>(smem + 2 * buf_bytes);   // [P][FZ_COLS + 1] segment bounds
    __shared__ T sh_rv[RES_CAP];
    __shared__ int32_t sh_rr[RES_CAP];
    __shared__ T sh_s[FZ_WAVES];
    __shared__ int64_t sh_c[FZ_WAVES];
    __shared__ T sh_out[FZ_COLS];          // largest |r| outside each column (found with the first value tile)
    // loads that depend on nothing go out first
    const int32_t done = st[0].done;
    const int32_t cnt = res_meta[RES_CNT];
    T rv_in = (T)-1;
    int32_t rr_in = -1;
    if (threadIdx.x < RES_CAP) { rv_in = res_val[threadIdx.x]; rr_in = res_row[threadIdx.x]; }
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int sub = lane & (ST_LPC - 1);
    const int rowid = lane / ST_LPC;
    const int32_t c0 = blockIdx.x * FZ_COLS;               // n < 2^31
    const int32_t ncol = n - c0 < FZ_COLS ? n - c0 : FZ_COLS;
    // The first trip to memory carries everything whose address is known now: partition 0 of r
    // (into registers; it is written to LDS below), this lane's segment bounds in partition 0
    // (straight into registers, so that its first entries can be requested without waiting for
    // the LDS table and a barrier), the table of all bounds, x and the reservoir.
    const bool aligned = (((size_t)mp * sizeof(T)) & 15) == 0;       // partitions start on 16 bytes
    const int32_t rows0 = (int32_t)(m < mp ? m : mp);
    const int32_t npiece0 = aligned ? (int32_t)(((size_t)rows0 * sizeof(T)) / 16) : 0;
    fz_piece rvp0[FZ_RV];
#pragma unroll
    for (int v = 0; v < FZ_RV; ++v) {
        const int32_t i = threadIdx.x + v * FZ_BLOCK;
        rvp0[v] = reinterpret_cast<const fz_piece*>(r)[i < npiece0 ? i : 0];
    }
    // the bounds of this workgroup's segments in every partition: one trip to memory for all of them
    for (int32_t t = threadIdx.x; t < P * (FZ_COLS + 1); t += FZ_BLOCK) {
        const int32_t p = t / (FZ_COLS + 1), cc = t - p * (FZ_COLS + 1);
        sh_seg[t] = cc <= ncol ? segptr[(int64_t)p * n + c0 + cc] : 0;
    }
    int32_t slot[FZ_GROUPS];               // column of the workgroup this lane works on, per group
    int32_t kcur[FZ_GROUPS];
    int32_t first_b0[FZ_GROUPS], first_b1[FZ_GROUPS];
    uint32_t flags = 0;                    // bit u: the column exists; bit 4 + u: it may move
#pragma unroll
    for (int u = 0; u < FZ_GROUPS; ++u) {
        slot[u] = (w + u * FZ_WAVES) * ST_CPW + rowid;
        const bool ok = slot[u] < ncol;
        const int32_t j = ok ? c0 + slot[u] : n - 1;
        kcur[u] = kidx[j];
        first_b0[u] = ok ? segptr[c0 + slot[u]] : 0;                 // partition 0
        first_b1[u] = ok ? segptr[c0 + slot[u] + 1] : SEG_ALIGN;
        const bool vok = var_mask ? var_mask[j] != 0 : true;
        flags |= (ok ? 1u : 0u) << u | (vok ? 1u : 0u) << (4 + u);
    }
    if (honor_done && done) return;
    T dcur[FZ_GROUPS];
#pragma unroll
    for (int u = 0; u < FZ_GROUPS; ++u) dcur[u] = D[kcur[u]];
    if (threadIdx.x < RES_CAP) {
        sh_rv[threadIdx.x] = (int32_t)threadIdx.x < cnt ? rv_in : (T)-1;
        sh_rr[threadIdx.x] = (int32_t)threadIdx.x < cnt ? rr_in : -1;
    }
    if (threadIdx.x == 0) { buf0[mp] = (T)0; buf1[mp] = (T)0; }      // what a pad's offset reads
    const int32_t nfast = cnt < RES_FAST ? cnt : RES_FAST;
    // partition 0 of r goes to LDS as soon as it arrives (its loads were the first issued, so
    // nothing requested later is held up by waiting for them, and their registers are free again)
#pragma unroll
    for (int v = 0; v < FZ_RV; ++v) {
        const int32_t i = threadIdx.x + v * FZ_BLOCK;
        if (i < npiece0) reinterpret_cast<fz_piece*>(buf0)[i] = rvp0[v];
    }

    T bs = (T)0;                 // this lane's best candidate so far
    int64_t bc = -1;

    // Per group: the two groups of four of the partition about to be folded (ix, av), this
    // lane's first entry of that segment and the segment's end (qe, qs1).  One spare group of
    // four per wavefront (`ext`), owned by group ext_owner (-1: free).
    uint2 ix[FZ_GROUPS][FZ_NQ];
    typename Vec4<T>::type av[FZ_GROUPS][FZ_NQ];
    int32_t qe[FZ_GROUPS], qs1[FZ_GROUPS];
    uint2 ext_ix;
    typename Vec4<T>::type ext_av;
    int32_t ext_owner = -1;
    // request the entries of group u in partition pp (a column that does not exist: entries 0..3, unused)
#define FZ_REQUEST(u, pp)                                                                              \
    do {                                                                                           \
        const bool ok_ = (flags >> (u)) & 1u;                                                      \
        FZ_REQUEST_B(u, ok_ ? sh_seg[(pp) * (FZ_COLS + 1) + slot[u]] : 0,                          \
                     ok_ ? sh_seg[(pp) * (FZ_COLS + 1) + slot[u] + 1] : SEG_ALIGN);                \
    } while (0)
#define FZ_REQUEST_B(u, lo_, hi_)                                                                      \
    do {                                                                                           \
        const int32_t b0_ = (lo_);                                                                 \
        const int32_t b1_ = (hi_);                                                                 \
        qe[u] = b0_ + sub * SEG_ALIGN;                                                             \
        qs1[u] = b1_;                                                                              \
        fz_load_quad<T>(ix[u][0], av[u][0], row16, cval, qe[u], b1_);                              \
        fz_load_quad<T>(ix[u][1], av[u][1], row16, cval, qe[u] + FZ_QSTEP, b1_);                   \
        if (ext_owner < 0 && __any(b1_ - b0_ > FZ_NQ * FZ_QSTEP)) {                                \
            ext_owner = (u);                                                                       \
            fz_load_quad<T>(ext_ix, ext_av, row16, cval, qe[u] + FZ_NQ * FZ_QSTEP, b1_);           \
        }                                                                                          \
    } while (0)
    // first value tile: its bounds were requested at the top of the kernel
#pragma unroll
    for (int u = 0; u < FZ_GROUPS; ++u) FZ_REQUEST_B(u, first_b0[u], first_b1[u]);

    for (int32_t k0 = 0; k0 < nd; k0 += KT) {
        T dk[KT], acc[FZ_GROUPS][KT];
        uint32_t mask[FZ_GROUPS];
#pragma unroll
        for (int q = 0; q < KT; ++q) dk[q] = D[k0 + q < nd ? k0 + q : nd - 1];
#pragma unroll
        for (int u = 0; u < FZ_GROUPS; ++u) {
            mask[u] = 0;
#pragma unroll
            for (int q = 0; q < KT; ++q) acc[u][q] = (T)0;
        }
        // ---- prologue: entries of partition 0, r of partition 0
        if (k0 > 0) {                     // (the first tile's requests went out before the loop)
#pragma unroll
            for (int u = 0; u < FZ_GROUPS; ++u) FZ_REQUEST(u, 0);
            for (int32_t i = threadIdx.x; i < npiece0; i += FZ_BLOCK)
                reinterpret_cast<fz_piece*>(buf0)[i] = reinterpret_cast<const fz_piece*>(r)[i];
        }
        for (int32_t i = npiece0 * (int32_t)(16 / sizeof(T)) + threadIdx.x; i < rows0; i += FZ_BLOCK) buf0[i] = r[i];
        __syncthreads();                  // partition 0 of r, the table of bounds and the reservoir are in place
        const T thr = nfast > 0 ? sh_rv[nfast - 1] : Limits<T>::inf();
        for (int32_t p = 0; p < P; ++p) {
            T* const cur = (p & 1) ? buf1 : buf0;
            T* const nxt = (p & 1) ? buf0 : buf1;
            const int64_t row0 = (int64_t)p * mp;
            const int32_t rows_here = (int32_t)((m - row0) < mp ? (m - row0) : mp);
            const int64_t row0n = row0 + mp;
            const int32_t rows_next = p + 1 < P ? (int32_t)((m - row0n) < mp ? (m - row0n) : mp) : 0;
            // partition p + 1 of r: requested now, written to the other buffer after the folds
            // (unconditional loads: a piece past the end repeats piece 0; no next partition: r itself)
            const int32_t npiece = aligned ? (int32_t)(((size_t)rows_next * sizeof(T)) / 16) : 0;
            fz_piece rvp[FZ_RV];
            {
                const fz_piece* __restrict__ src = reinterpret_cast<const fz_piece*>(npiece > 0 ? r + row0n : r);
#pragma unroll
                for (int v = 0; v < FZ_RV; ++v) {
                    const int32_t i = threadIdx.x + v * FZ_BLOCK;
                    rvp[v] = src[i < npiece ? i : 0];
                }
            }
#pragma unroll
            for (int u = 0; u < FZ_GROUPS; ++u) {
                fz_fold_quad<T, KT>(ix[u][0], av[u][0], cur, dk, dcur[u], acc[u], mask[u], k0 == 0, thr, nfast, sh_rr, row0, rows_here);
                fz_fold_quad<T, KT>(ix[u][1], av[u][1], cur, dk, dcur[u], acc[u], mask[u], k0 == 0, thr, nfast, sh_rr, row0, rows_here);
                int32_t e = qe[u] + FZ_NQ * FZ_QSTEP;
                if (ext_owner == u) {
                    fz_fold_quad<T, KT>(ext_ix, ext_av, cur, dk, dcur[u], acc[u], mask[u], k0 == 0, thr, nfast, sh_rr, row0, rows_here);
                    e += FZ_QSTEP;
                    ext_owner = -1;
                }
                // what is left of long segments: loads that are waited for (the columns diverge here)
                const int32_t seg_end = qs1[u];
                for (; e - sub * SEG_ALIGN < seg_end; e += FZ_QSTEP) {
                    uint2 lix;
                    typename Vec4<T>::type lav;
                    fz_load_quad<T>(lix, lav, row16, cval, e, seg_end);
                    fz_fold_quad<T, KT>(lix, lav, cur, dk, dcur[u], acc[u], mask[u], k0 == 0, thr, nfast, sh_rr, row0, rows_here);
                }
                if (p + 1 < P) FZ_REQUEST(u, p + 1);       // these registers take the next partition
            }
            if (p + 1 < P) {
#pragma unroll
                for (int v = 0; v < FZ_RV; ++v) {
                    const int32_t i = threadIdx.x + v * FZ_BLOCK;
                    if (i < npiece) reinterpret_cast<fz_piece*>(nxt)[i] = rvp[v];
                }
                for (int32_t i = npiece * (int32_t)(16 / sizeof(T)) + threadIdx.x; i < rows_next; i += FZ_BLOCK) nxt[i] = r[row0n + i];
            }
            __syncthreads();                  // partition p consumed by all, partition p + 1 in place
        }
#undef FZ_REQUEST
#undef FZ_REQUEST_B
        // ---- the columns' scores: partition maxima are complete, add the rows outside the column
#pragma unroll
        for (int u = 0; u < FZ_GROUPS; ++u) {
#pragma unroll
            for (int q = 0; q < KT; ++q) acc[u][q] = lanes_max_nonneg<ST_LPC>(acc[u][q]);
            const bool ok = (flags >> u) & 1u;
            const int32_t j = ok ? c0 + slot[u] : n - 1;
            T outside_u;
            if (k0 == 0) {
                outside_u = (T)0;
                const uint32_t cm = lanes_or<ST_LPC>(mask[u]);
                const uint32_t full = (1u << nfast) - 1u;          // RES_FAST < 32
                const uint32_t missing = full & ~cm;
                bool need_walk = false;
                if (missing) outside_u = sh_rv[__builtin_ctz(missing)];
                else if ((int64_t)nfast >= m) outside_u = (T)0;    // the column holds every row
                else need_walk = ok;
                // rare: the column contains every inline-checked reservoir row; the wavefront helps
                unsigned long long todo = __ballot(need_walk && sub == 0);
                while (todo) {
                    const int src = __builtin_ctzll(todo);
                    todo &= todo - 1;
                    const int64_t jj = __shfl(j, src, 64);
                    int32_t first = INT32_MAX;
                    for (int32_t base = RES_FAST; base < cnt && first == INT32_MAX; base += 64) {
                        const int32_t q = base + lane;
                        const bool absent = q < cnt && !column_has_row<T>(segptr, row16, n, mp, jj, sh_rr[q]);
                        const unsigned long long bal = __ballot(absent);
                        if (bal) first = base + __builtin_ctzll(bal);
                    }
                    T o;
                    if (first != INT32_MAX) {
                        o = sh_rv[first];
                    } else if ((int64_t)cnt >= m) {
                        o = (T)0;
                    } else {                                       // exact scan over all rows
                        o = (T)0;
                        for (int64_t i = lane; i < m; i += 64)
                            if (!column_has_row<T>(segptr, row16, n, mp, jj, (int32_t)i)) o = dmmv_max(o, dmmv_abs(r[i]));
                        o = wave_max(o);
                    }
                    if ((lane & ~(ST_LPC - 1)) == (src & ~(ST_LPC - 1))) outside_u = o;   // the column's lanes
                }
                if (sub == 0 && nd > KT) sh_out[slot[u]] = outside_u;   // later value tiles read it back (same lane)
            } else {
                outside_u = sh_out[slot[u]];
            }
            // every lane of the column holds the column's maxima: lane `sub` scores value k0 + sub
            static_assert(KT <= ST_LPC, "one lane of the column per value of the tile");
            T mine = acc[u][0];
#pragma unroll
            for (int q = 1; q < KT; ++q) mine = sub == q ? acc[u][q] : mine;
            const int32_t k = k0 + sub;
            if (ok && sub < KT && k < nd) {
                const bool vok = (flags >> (4 + u)) & 1u;
                T v = dmmv_max(outside_u, mine);
                if (!cand_allowed(kcur[u], k, radius, vok)) v = Limits<T>::inf();
                const int64_t cidx = (int64_t)j * nd + k;
                if (scores) scores[cidx] = v;
                if (rec_less(v, cidx, bs, bc)) { bs = v; bc = cidx; }
            }
        }
    }
    if (part) {
        block_argmin(bs, bc, sh_s, sh_c);
        if (threadIdx.x == 0) { Partial<T> pr; pr.s = bs; pr.c = bc; part[blockIdx.x] = pr; }
    }
}

// =========================================================================================
// finalize
// =========================================================================================
template <class T>
__global__ __launch_bounds__(FIN_BLOCK) void k_finalize_csc(
    int64_t m, int64_t n, int32_t nd, int32_t mp, int32_t P, const int32_t* __restrict__ segptr,
    const uint16_t* __restrict__ row16, const int32_t* __restrict__ kidx, const T* __restrict__ r,
    const T* __restrict__ res_val, const int32_t* __restrict__ res_row,
    const int32_t* __restrict__ res_meta, const T* __restrict__ part_scores,
    const uint32_t* __restrict__ part_mask, int32_t radius, const uint8_t* __restrict__ var_mask,
    const InstState<T>* __restrict__ st, int32_t honor_done, T* __restrict__ scores,
    Partial<T>* __restrict__ part) {
    constexpr int KPF = 8;                                 // values of D whose partition maxima are fetched up front
    __shared__ T sh_rv[RES_CAP];
    __shared__ int32_t sh_rr[RES_CAP];
    __shared__ T sh_s[FIN_BLOCK / 64];
    __shared__ int64_t sh_c[FIN_BLOCK / 64];
    const int lane = threadIdx.x & 63;
    const int64_t j = blockIdx.x * (int64_t)FIN_BLOCK + threadIdx.x;
    const bool live = j < n;
    const int64_t jc = live ? j : n - 1;
    // Every global load that does not depend on another is issued here, before the first
    // wait: the stop flag, the reservoir, the column's masks, its current value and the
    // partition maxima of its first KPF values.  The kernel is a chain of memory latencies
    // otherwise.
    const int32_t done = st[0].done;
    const int32_t cnt = res_meta[RES_CNT];
    T rv = (T)-1;
    int32_t rr = -1;
    if (threadIdx.x < RES_CAP) { rv = res_val[threadIdx.x]; rr = res_row[threadIdx.x]; }
    uint32_t cm = 0;
    for (int32_t p = 0; p < P; ++p) cm |= part_mask[(int64_t)p * n + jc];
    const int32_t kcur = kidx[jc];
    T pmax[KPF];
#pragma unroll
    for (int k = 0; k < KPF; ++k) {
        pmax[k] = (T)0;
        if (k < nd)
            for (int32_t p = 0; p < P; ++p)
                pmax[k] = dmmv_max(pmax[k], part_scores[(int64_t)p * (n * (int64_t)nd) + jc * (int64_t)nd + k]);
    }
    if (honor_done && done) return;
    if (threadIdx.x < RES_CAP) {
        sh_rv[threadIdx.x] = (int32_t)threadIdx.x < cnt ? rv : (T)-1;
        sh_rr[threadIdx.x] = (int32_t)threadIdx.x < cnt ? rr : -1;
    }
    __syncthreads();
    const int32_t nfast = cnt < RES_FAST ? cnt : RES_FAST;
    const uint32_t full = (1u << nfast) - 1u;              // RES_FAST < 32

    T outside = (T)0;
    bool need_walk = false;
    if (live) {
        const uint32_t missing = full & ~cm;
        if (missing) outside = sh_rv[__builtin_ctz(missing)];
        else if ((int64_t)nfast >= m) outside = (T)0;          // the column holds every row
        else need_walk = true;
    }
    // rare: the column contains every inline-checked reservoir row; the whole wavefront helps
    unsigned long long todo = __ballot(need_walk);
    while (todo) {
        const int src = __builtin_ctzll(todo);
        todo &= todo - 1;
        const int64_t jj = __shfl(j, src, 64);
        // 1) the rest of the reservoir, in order: first entry whose row is not in the column
        int32_t first = INT32_MAX;
        for (int32_t base = RES_FAST; base < cnt && first == INT32_MAX; base += 64) {
            const int32_t q = base + lane;
            const bool absent = q < cnt && !column_has_row<T>(segptr, row16, n, mp, jj, sh_rr[q]);
            const unsigned long long b = __ballot(absent);
            if (b) first = base + __builtin_ctzll(b);
        }
        T o;
        if (first != INT32_MAX) {
            o = sh_rv[first];
        } else if ((int64_t)cnt >= m) {
            o = (T)0;
        } else {
            // 2) exact scan over all rows
            o = (T)0;
            for (int64_t i = lane; i < m; i += 64)
                if (!column_has_row<T>(segptr, row16, n, mp, jj, (int32_t)i)) o = dmmv_max(o, dmmv_abs(r[i]));
            o = wave_max(o);
        }
        if (lane == src) outside = o;
    }

    T bs = (T)0;
    int64_t bc = -1;
    if (live) {
        const bool var_ok = var_mask ? var_mask[j] != 0 : true;
        for (int32_t k = 0; k < nd; ++k) {
            const int64_t cidx = j * (int64_t)nd + k;
            T v = outside;
            if (k < KPF) {
                T pm = pmax[0];
#pragma unroll
                for (int q = 1; q < KPF; ++q) pm = k == q ? pmax[q] : pm;
                v = dmmv_max(v, pm);
            } else {
                for (int32_t p = 0; p < P; ++p) v = dmmv_max(v, part_scores[(int64_t)p * (n * (int64_t)nd) + cidx]);
            }
            if (!cand_allowed(kcur, k, radius, var_ok)) v = Limits<T>::inf();
            if (scores) scores[cidx] = v;
            if (rec_less(v, cidx, bs, bc)) { bs = v; bc = cidx; }
        }
    }
    if (part) {
        block_argmin(bs, bc, sh_s, sh_c);
        if (threadIdx.x == 0) { Partial<T> pr; pr.s = bs; pr.c = bc; part[blockIdx.x] = pr; }
    }
}

// =========================================================================================
// pruned evaluation (for the descent, where only a strictly improving move matters)
// =========================================================================================
// A move improves only if it lowers EVERY row whose |r| equals the current maximum t; a row
// that has no entry in column j is not changed by moving x_j.  So only the columns with an
// entry in the row i* of largest |r| (the head of the reservoir) can hold an improving move.
// One wavefront per entry of row i* scores that column exactly as the full evaluation does
// (all its entries, plus the maximum over the rows outside the column) and writes one arg-min
// record.  If an improving move exists, the arg-min over these records is the arg-min over the
// whole table; if none exists, the best record is not an improvement either, and the loop
// stops just the same.
template <class T>
__global__ __launch_bounds__(64) void k_eval_pruned_csc(
    int64_t m, int64_t n, int32_t nd, int32_t mp, int32_t P, const int64_t* __restrict__ csr_rowptr,
    const int32_t* __restrict__ csr_col, const int32_t* __restrict__ segptr,
    const uint16_t* __restrict__ row16, const T* __restrict__ cval, const T* __restrict__ D,
    const int32_t* __restrict__ kidx, const T* __restrict__ r, const T* __restrict__ res_val,
    const int32_t* __restrict__ res_row, const int32_t* __restrict__ res_meta, int32_t radius,
    const uint8_t* __restrict__ var_mask, const InstState<T>* __restrict__ st, int32_t honor_done,
    Partial<T>* __restrict__ part) {
    constexpr int KT = 8;
    if (honor_done && st[0].done) return;
    const int lane = threadIdx.x;
    Partial<T> rec; rec.s = (T)0; rec.c = -1;
    const int32_t cnt = res_meta[RES_CNT];
    int64_t j = -1;
    if (cnt > 0) {
        const int64_t istar = res_row[0];
        const int64_t e = csr_rowptr[istar] + blockIdx.x;
        if (e < csr_rowptr[istar + 1]) j = csr_col[e];
    }
    if (j < 0) {                                   // no such entry: an empty record
        if (lane == 0) part[blockIdx.x] = rec;
        return;
    }
    // maximum over the rows outside column j: first reservoir row the column does not hold
    T outside = (T)0;
    {
        int32_t first = INT32_MAX;
        for (int32_t base = 0; base < cnt && first == INT32_MAX; base += 64) {
            const int32_t q = base + lane;
            const bool absent = q < cnt && !column_has_row<T>(segptr, row16, n, mp, j, res_row[q]);
            const unsigned long long b = __ballot(absent);
            if (b) first = base + __builtin_ctzll(b);
        }
        if (first != INT32_MAX) {
            outside = res_val[first];
        } else if ((int64_t)cnt < m) {             // the column holds the whole reservoir: exact scan
            T o = (T)0;
            for (int64_t i = lane; i < m; i += 64)
                if (!column_has_row<T>(segptr, row16, n, mp, j, (int32_t)i)) o = dmmv_max(o, dmmv_abs(r[i]));
            outside = wave_max(o);
        }
    }
    const int32_t kcur = kidx[j];
    const T dcur = D[kcur];
    const bool var_ok = var_mask ? var_mask[j] != 0 : true;
    for (int32_t k0 = 0; k0 < nd; k0 += KT) {
        T delta[KT], acc[KT];
#pragma unroll
        for (int q = 0; q < KT; ++q) {
            delta[q] = step_of(D[k0 + q < nd ? k0 + q : nd - 1], dcur, (T)1);
            acc[q] = (T)0;
        }
        for (int32_t p = 0; p < P; ++p) {
            const int32_t e0 = segptr[(int64_t)p * n + j], e1 = segptr[(int64_t)p * n + j + 1];
            for (int32_t e = e0 + lane; e < e1; e += 64) {
                const uint32_t loc = row16[e];
                if (loc == (uint32_t)mp) continue;
                const T a = cval[e], ri = r[(int64_t)p * mp + loc];
#pragma unroll
                for (int q = 0; q < KT; ++q) acc[q] = dmmv_max(acc[q], dmmv_abs(dmmv_fma(delta[q], a, ri)));
            }
        }
#pragma unroll
        for (int q = 0; q < KT; ++q) {
            const int32_t k = k0 + q;
            T v = dmmv_max(wave_max(acc[q]), outside);
            if (k < nd) {
                if (!cand_allowed(kcur, k, radius, var_ok)) v = Limits<T>::inf();
                const int64_t cidx = j * (int64_t)nd + k;
                if (rec_less(v, cidx, rec.s, rec.c)) { rec.s = v; rec.c = cidx; }
            }
        }
    }
    if (lane == 0) part[blockIdx.x] = rec;
}

// The same records with fewer trips to memory, for columns of at most 64 * PR_SLOTS entries
// (padding included).  The kernel above is a chain of some fourteen dependent accesses (row of
// largest |r| -> its entries -> segment bounds -> binary searches for the reservoir rows ->
// current value -> entries -> residuals); a wavefront that has nothing else to do pays each of
// them in full.  Here a lane keeps up to PR_SLOTS entries of the column (row, value, residual)
// and two reservoir rows in registers, so whether a reservoir row is in the column is a
// comparison across lanes, and what remains is six dependent accesses.
constexpr int PR_SLOTS = 8;

template <class T>
__global__ __launch_bounds__(64) void k_eval_pruned_csc_reg(
    int64_t m, int64_t n, int32_t nd, int32_t mp, int32_t P, const int64_t* __restrict__ csr_rowptr,
    const int32_t* __restrict__ csr_col, const int32_t* __restrict__ segptr,
    const uint16_t* __restrict__ row16, const T* __restrict__ cval, const T* __restrict__ D,
    const int32_t* __restrict__ kidx, const T* __restrict__ r, const T* __restrict__ res_val,
    const int32_t* __restrict__ res_row, const int32_t* __restrict__ res_meta, int32_t radius,
    const uint8_t* __restrict__ var_mask, const InstState<T>* __restrict__ st, int32_t honor_done,
    Partial<T>* __restrict__ part) {
    constexpr int KT = 8;
    static_assert(RES_CAP <= 128, "two reservoir entries per lane");
    const int lane = threadIdx.x;
    // 1: everything that depends on nothing
    const int32_t done = st[0].done;
    const int32_t cnt = res_meta[RES_CNT];
    const int32_t rr0 = res_row[lane], rr1 = res_row[lane + 64];      // RES_CAP = 128 entries exist
    const T rv0 = res_val[lane], rv1 = res_val[lane + 64];
    // the levels travel with these loads when they fit the lanes (lane k holds D[k]); later reads
    // of a level are lane reads, not trips to memory
    const bool d_in_lanes = nd <= 64;
    const T d_lane = D[lane < nd ? lane : nd - 1];
    if (honor_done && done) return;
    Partial<T> rec; rec.s = (T)0; rec.c = -1;
    int64_t j = -1;
    if (cnt > 0) {
        const int64_t istar = __builtin_amdgcn_readfirstlane(rr0);
        const int64_t e = csr_rowptr[istar] + blockIdx.x;                   // 2
        if (e < csr_rowptr[istar + 1]) j = csr_col[e];                      // 3
    }
    if (j < 0) {                                   // no such entry: an empty record
        if (lane == 0) part[blockIdx.x] = rec;
        return;
    }
    // 4: the segment bounds and the current value; a lane's slots are entries lane, lane + 64, ...
    // (up to 64 partitions: lane p fetches the bounds of partition p, all in one trip)
    const int32_t kcur = __builtin_amdgcn_readfirstlane(kidx[j]);
    int32_t ent[PR_SLOTS], part_of[PR_SLOTS];
#pragma unroll
    for (int u = 0; u < PR_SLOTS; ++u) { ent[u] = -1; part_of[u] = 0; }
    {
        const bool by_lane = P <= 64;
        int32_t my_e0 = 0, my_len = 0;
        if (by_lane && lane < P) {
            my_e0 = segptr[(int64_t)lane * n + j];
            my_len = segptr[(int64_t)lane * n + j + 1] - my_e0;
        }
        int32_t base = 0;
        for (int32_t p = 0; p < P; ++p) {
            int32_t e0, len;
            if (by_lane) {
                e0 = __builtin_amdgcn_readlane(my_e0, p);
                len = __builtin_amdgcn_readlane(my_len, p);
            } else {
                e0 = segptr[(int64_t)p * n + j];
                len = segptr[(int64_t)p * n + j + 1] - e0;
            }
#pragma unroll
            for (int u = 0; u < PR_SLOTS; ++u) {
                const int32_t t = lane + 64 * u - base;
                if (t >= 0 && t < len) { ent[u] = e0 + t; part_of[u] = p; }
            }
            base += len;
        }
    }
    // 5: entries, current value of D;  6: residuals
    int32_t row[PR_SLOTS];
    T a[PR_SLOTS], ri[PR_SLOTS];
#pragma unroll
    for (int u = 0; u < PR_SLOTS; ++u) {
        row[u] = -1;
        a[u] = (T)0;
        if (ent[u] >= 0) {
            const uint32_t loc = row16[ent[u]];
            if (loc != (uint32_t)mp) { row[u] = part_of[u] * mp + (int32_t)loc; a[u] = cval[ent[u]]; }
        }
    }
    const T dcur = d_in_lanes ? read_lane(d_lane, kcur) : D[kcur];
#pragma unroll
    for (int u = 0; u < PR_SLOTS; ++u) ri[u] = row[u] >= 0 ? r[row[u]] : (T)0;
    // maximum over the rows outside column j: first reservoir row the column does not hold
    T outside = (T)0;
    {
        int32_t first = -1;
        for (int32_t q = 0; q < cnt; ++q) {
            const int32_t want = q < 64 ? __builtin_amdgcn_readlane(rr0, q) : __builtin_amdgcn_readlane(rr1, q - 64);
            bool hit = false;
#pragma unroll
            for (int u = 0; u < PR_SLOTS; ++u) hit = hit || row[u] == want;
            if (!__any(hit)) { first = q; break; }
        }
        if (first >= 0) {
            outside = first < 64 ? read_lane(rv0, first) : read_lane(rv1, first - 64);
        } else if ((int64_t)cnt < m) {             // the column holds the whole reservoir: exact scan
            T o = (T)0;
            for (int64_t i = lane; i < m; i += 64)
                if (!column_has_row<T>(segptr, row16, n, mp, j, (int32_t)i)) o = dmmv_max(o, dmmv_abs(r[i]));
            outside = wave_max(o);
        }
    }
    const bool var_ok = var_mask ? var_mask[j] != 0 : true;
    for (int32_t k0 = 0; k0 < nd; k0 += KT) {
        T delta[KT], acc[KT];
#pragma unroll
        for (int q = 0; q < KT; ++q) {
            const int32_t kq = k0 + q < nd ? k0 + q : nd - 1;
            delta[q] = step_of(d_in_lanes ? read_lane(d_lane, kq) : D[kq], dcur, (T)1);
            acc[q] = (T)0;
        }
#pragma unroll
        for (int u = 0; u < PR_SLOTS; ++u)
            if (row[u] >= 0) {
#pragma unroll
                for (int q = 0; q < KT; ++q) acc[q] = dmmv_max(acc[q], dmmv_abs(dmmv_fma(delta[q], a[u], ri[u])));
            }
#pragma unroll
        for (int q = 0; q < KT; ++q) {
            const int32_t k = k0 + q;
            T v = dmmv_max(wave_max(acc[q]), outside);
            if (k < nd) {
                if (!cand_allowed(kcur, k, radius, var_ok)) v = Limits<T>::inf();
                const int64_t cidx = j * (int64_t)nd + k;
                if (rec_less(v, cidx, rec.s, rec.c)) { rec.s = v; rec.c = cidx; }
            }
        }
    }
    if (lane == 0) part[blockIdx.x] = rec;
}

// =========================================================================================
// host dispatch
// =========================================================================================
template <class T, int KT>
static dmmv_status stream_launch(Ctx* c, bool honor_done) {
    if (c->csc_P > CSC_MAX_PARTITIONS)
        return fail(DMMV_ERR_UNSUPPORTED, "sparse path: %d row partitions exceed the limit of %d (raise sparse_partition_rows)", c->csc_P, CSC_MAX_PARTITIONS);
    const size_t lds = ((size_t)c->csc_mp + 1) * sizeof(T);
    DMMV_TRY(ensure_dynamic_lds(reinterpret_cast<const void*>(&k_eval_stream<T, KT>), CSC_LDS_BYTES + 256));
    dim3 grid((unsigned)c->csc_gb, (unsigned)c->csc_P);
    hipLaunchKernelGGL((k_eval_stream<T, KT>), grid, dim3(ST_BLOCK), lds, c->stream, c->p.m, c->p.n,
                       c->p.nd, c->csc_mp, (const int32_t*)c->segptr, (const uint16_t*)c->row16,
                       (const T*)c->cval, (const int32_t*)c->blk_lo, (const T*)c->D_dev,
                       (const int32_t*)c->kidx, (const T*)c->r, (const T*)c->res_val,
                       (const int32_t*)c->res_row, (const int32_t*)c->res_meta,
                       (const InstState<T>*)c->state, (int32_t)honor_done, (T*)c->part_scores,
                       c->part_mask);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status stream_t(Ctx* c, bool honor_done) {
    if (c->p.nd <= 2) return stream_launch<T, 2>(c, honor_done);
    if (c->p.nd == 3) return stream_launch<T, 3>(c, honor_done);
    if (c->p.nd <= 4) return stream_launch<T, 4>(c, honor_done);
    return stream_launch<T, 8>(c, honor_done);
}

template <class T, int KT>
static dmmv_status fused_launch(Ctx* c, void* scores, bool want_partials, bool honor_done) {
    const size_t buf = (((size_t)c->csc_mp + 1) * sizeof(T) + 15) / 16 * 16;
    const size_t lds = 2 * buf + (size_t)c->csc_P * (FZ_COLS + 1) * sizeof(int32_t);
    if (c->csc_P > FZ_MAX_P) return fail(DMMV_ERR_STATE, "one-kernel sparse evaluation chosen for %d partitions (at most %d)", c->csc_P, FZ_MAX_P);
    DMMV_TRY(ensure_dynamic_lds(reinterpret_cast<const void*>(&k_eval_fused<T, KT>),
                                2 * CSC_LDS_BYTES + 64 + FZ_MAX_P * (FZ_COLS + 1) * (int)sizeof(int32_t)));
    const unsigned blocks = (unsigned)ceil_div(c->p.n, FZ_COLS);
    if ((int64_t)blocks != c->n_partials) return fail(DMMV_ERR_STATE, "sparse evaluation grid does not match the partial-record buffer");
    hipLaunchKernelGGL((k_eval_fused<T, KT>), dim3(blocks), dim3(FZ_BLOCK), lds, c->stream, c->p.m, (int32_t)c->p.n,
                       c->p.nd, c->csc_mp, c->csc_P, (const int32_t*)c->segptr, (const uint16_t*)c->row16,
                       (const T*)c->cval, (const T*)c->D_dev, (const int32_t*)c->kidx, (const T*)c->r,
                       (const T*)c->res_val, (const int32_t*)c->res_row, (const int32_t*)c->res_meta,
                       (const InstState<T>*)c->state, (int32_t)honor_done, c->o.radius, c->o.var_mask,
                       (T*)scores, want_partials ? (Partial<T>*)c->partials : nullptr);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

template <class T>
static dmmv_status eval_t(Ctx* c, void* scores, bool want_partials, bool honor_done) {
    if (c->csc_fused) {
        if (c->p.nd <= 2) return fused_launch<T, 2>(c, scores, want_partials, honor_done);
        if (c->p.nd == 3) return fused_launch<T, 3>(c, scores, want_partials, honor_done);
        if (c->p.nd <= 4) return fused_launch<T, 4>(c, scores, want_partials, honor_done);
        return fused_launch<T, 8>(c, scores, want_partials, honor_done);
    }
    DMMV_TRY(stream_t<T>(c, honor_done));
    const unsigned blocks = (unsigned)ceil_div(c->p.n, FIN_BLOCK);
    if ((int64_t)blocks != c->n_partials) return fail(DMMV_ERR_STATE, "sparse finalize grid does not match the partial-record buffer");
    hipLaunchKernelGGL(k_finalize_csc<T>, dim3(blocks), dim3(FIN_BLOCK), 0, c->stream, c->p.m, c->p.n,
                       c->p.nd, c->csc_mp, c->csc_P, (const int32_t*)c->segptr, (const uint16_t*)c->row16,
                       (const int32_t*)c->kidx, (const T*)c->r, (const T*)c->res_val,
                       (const int32_t*)c->res_row, (const int32_t*)c->res_meta,
                       (const T*)c->part_scores, (const uint32_t*)c->part_mask, c->o.radius,
                       c->o.var_mask, (const InstState<T>*)c->state, (int32_t)honor_done, (T*)scores,
                       want_partials ? (Partial<T>*)c->partials : nullptr);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}

dmmv_status csc_eval(Ctx* c, void* scores_out, bool want_partials, bool honor_done) {
    return c->p.dtype == DMMV_F64 ? eval_t<double>(c, scores_out, want_partials, honor_done)
                                  : eval_t<float>(c, scores_out, want_partials, honor_done);
}
template <class T>
static dmmv_status eval_pruned_t(Ctx* c, bool honor_done) {
    if (c->csc_max_row <= 0) return DMMV_OK;       // no stored entry anywhere: nothing can move r
    // short columns: the variant that keeps the column in registers
    auto kernel = c->csc_max_col <= 64 * PR_SLOTS ? k_eval_pruned_csc_reg<T> : k_eval_pruned_csc<T>;
    hipLaunchKernelGGL(kernel, dim3((unsigned)c->csc_max_row), dim3(64), 0, c->stream, c->p.m,
                       c->p.n, c->p.nd, c->csc_mp, c->csc_P, c->p.csr_rowptr, c->p.csr_col,
                       (const int32_t*)c->segptr, (const uint16_t*)c->row16, (const T*)c->cval,
                       (const T*)c->D_dev, (const int32_t*)c->kidx, (const T*)c->r, (const T*)c->res_val,
                       (const int32_t*)c->res_row, (const int32_t*)c->res_meta, c->o.radius, c->o.var_mask,
                       (const InstState<T>*)c->state, (int32_t)honor_done, (Partial<T>*)c->prune_part);
    DMMV_LAUNCH_CHECK();
    return DMMV_OK;
}
dmmv_status csc_eval_pruned(Ctx* c, bool honor_done) {
    return c->p.dtype == DMMV_F64 ? eval_pruned_t<double>(c, honor_done) : eval_pruned_t<float>(c, honor_done);
}

}  // namespace dmmv
