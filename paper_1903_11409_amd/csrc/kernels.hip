// Device kernels of libbspmm for gfx950 (wave64).
//
// bspmm_kernel      one launch computes every work item of a schedule: per item, stage the
//                   operation's CSR arrays and the feature tile of its dense input in LDS
//                   (or, for the generic bin, read them from global memory), then give every
//                   output row a group of lanes that accumulates its stored entries in
//                   registers and writes the row once (the row-wise, atomic-free product of
//                   Fig. 4, batched as in Sec. IV-C, with the column blocking of Fig. 5(d)).
// build_transpose   stable CSR -> transposed CSR of every operation (counting sort by column).
// validate_csr      structural check of the device CSR arrays.
#include <hip/hip_runtime.h>

#include "plan.hpp"

namespace bspmm {

// ---------------------------------------------------------------------------------------
// small vector helpers
// ---------------------------------------------------------------------------------------
template <int VEC> struct Vec;
template <> struct Vec<4> {
    using type = float4;
    static __device__ __forceinline__ type zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
    static __device__ __forceinline__ void fma(type& acc, float a, const type& b)
    {
        acc.x = fmaf(a, b.x, acc.x);
        acc.y = fmaf(a, b.y, acc.y);
        acc.z = fmaf(a, b.z, acc.z);
        acc.w = fmaf(a, b.w, acc.w);
    }
};
template <> struct Vec<1> {
    using type = float;
    static __device__ __forceinline__ type zero() { return 0.f; }
    static __device__ __forceinline__ void fma(type& acc, float a, const type& b)
    {
        acc = fmaf(a, b, acc);
    }
};

template <int VEC>
__device__ __forceinline__ typename Vec<VEC>::type load_vec(const float* p)
{
    return *reinterpret_cast<const typename Vec<VEC>::type*>(p);
}
template <int VEC>
__device__ __forceinline__ void store_vec(float* p, const typename Vec<VEC>::type& v)
{
    *reinterpret_cast<typename Vec<VEC>::type*>(p) = v;
}

__device__ __forceinline__ int ilog2(int pow2) { return 31 - __clz(pow2); }

// How the S lanes of a slot split into row groups for a tile of fw columns.
template <int S, int VEC>
struct Split {
    int g_lanes;   // lanes per row (power of two, <= S and <= 64)
    int groups;    // rows in flight
    int g;         // this lane's row group
    int l;         // this lane's position inside the group
    int nvec;      // vectors per tile row
    __device__ __forceinline__ Split(int fw, int lane)
    {
        int gl = lanes_per_row(fw, VEC);
        if (gl > S) gl = S;
        g_lanes = gl;
        const int sh = ilog2(gl);
        groups = S >> sh;
        g = lane >> sh;
        l = lane & (gl - 1);
        nvec = (fw + VEC - 1) / VEC;
    }
};

// ---------------------------------------------------------------------------------------
// staging: global -> LDS.  The three copies (row pointers, entries, dense tile) do not depend
// on each other, and none depends on the contents of the CSR arrays.  What decides the time
// of a small item is the number of global-memory round trips on its critical path, so the
// first trip of every copy is issued before anything is waited for: one round trip stages a
// typical molecule-sized item completely; larger items finish in unrolled leftover loops.
// ---------------------------------------------------------------------------------------
template <int S, int VEC>
__device__ __forceinline__ void stage_item(const LaunchParams& P, const WorkItem& it, int* sm,
                                           int lane)
{
    using VT = typename Vec<VEC>::type;
    const StagedLayout L = staged_layout(it.m, it.k, it.nnz, it.fw, P.pad);
    const int32_t* __restrict__ rp = P.rpt + it.rpt_off;
    const int32_t* __restrict__ ci = P.colids + it.nz_off;
    const float* __restrict__ va = P.values + it.nz_off;
    int2* cv = reinterpret_cast<int2*>(sm + L.cv_off);
    float* bs = reinterpret_cast<float*>(sm + L.b_off);
    const float* __restrict__ src = P.in + it.in_row_off * P.ld_in + it.f0;
    const Split<S, VEC> sp(it.fw, lane);
    const int step = sp.groups;
    const int m = it.m, nnz = it.nnz, k = it.k;

    // ---- first trip of every copy: loads only
    int rv = 0;
    if (lane <= m) rv = rp[lane];
    int c0 = 0, c1 = 0;
    float a0 = 0.f, a1 = 0.f;
    if (lane < nnz) {
        c0 = ci[lane];
        a0 = va[lane];
    }
    if (lane + S < nnz) {
        c1 = ci[lane + S];
        a1 = va[lane + S];
    }
    const bool col_ok = sp.l < sp.nvec;
    const int r0 = sp.g, r1 = sp.g + step, r2 = sp.g + 2 * step, r3 = sp.g + 3 * step;
    const float* colp = src + sp.l * VEC;
    VT t0 = Vec<VEC>::zero(), t1 = Vec<VEC>::zero(), t2 = Vec<VEC>::zero(), t3 = Vec<VEC>::zero();
    if (col_ok && r0 < k) t0 = load_vec<VEC>(colp + (int64_t)r0 * P.ld_in);
    if (col_ok && r1 < k) t1 = load_vec<VEC>(colp + (int64_t)r1 * P.ld_in);
    if (col_ok && r2 < k) t2 = load_vec<VEC>(colp + (int64_t)r2 * P.ld_in);
    if (col_ok && r3 < k) t3 = load_vec<VEC>(colp + (int64_t)r3 * P.ld_in);

    // ---- first trip: LDS writes.  Row pointers are clamped to [0, nnz] and columns to
    // [0, k) so that malformed arrays cannot make a lane leave its slot.
    if (lane <= m) sm[lane] = min(max(rv, 0), nnz);
    if (lane < nnz) cv[lane] = make_int2((unsigned)c0 < (unsigned)k ? c0 : 0, __float_as_int(a0));
    if (lane + S < nnz)
        cv[lane + S] = make_int2((unsigned)c1 < (unsigned)k ? c1 : 0, __float_as_int(a1));
    float* bcol = bs + sp.l * VEC;
    if (col_ok && r0 < k) store_vec<VEC>(bcol + r0 * L.stride, t0);
    if (col_ok && r1 < k) store_vec<VEC>(bcol + r1 * L.stride, t1);
    if (col_ok && r2 < k) store_vec<VEC>(bcol + r2 * L.stride, t2);
    if (col_ok && r3 < k) store_vec<VEC>(bcol + r3 * L.stride, t3);

    // ---- leftovers of larger items
    for (int i = lane + S; i <= m; i += S) sm[i] = min(max(rp[i], 0), nnz);
    for (int p = lane + 2 * S; p < nnz; p += 2 * S) {
        const int q = p + S;
        const int cc0 = ci[p];
        const float aa0 = va[p];
        int cc1 = 0;
        float aa1 = 0.f;
        if (q < nnz) {
            cc1 = ci[q];
            aa1 = va[q];
        }
        cv[p] = make_int2((unsigned)cc0 < (unsigned)k ? cc0 : 0, __float_as_int(aa0));
        if (q < nnz) cv[q] = make_int2((unsigned)cc1 < (unsigned)k ? cc1 : 0, __float_as_int(aa1));
    }
    for (int v = sp.l; v < sp.nvec; v += sp.g_lanes) {
        const float* cp = src + v * VEC;
        float* bp = bs + v * VEC;
        for (int row = (v == sp.l ? sp.g + 4 * step : sp.g); row < k; row += 4 * step) {
            const int q1 = row + step, q2 = row + 2 * step, q3 = row + 3 * step;
            VT u0 = load_vec<VEC>(cp + (int64_t)row * P.ld_in);
            VT u1 = Vec<VEC>::zero(), u2 = Vec<VEC>::zero(), u3 = Vec<VEC>::zero();
            if (q1 < k) u1 = load_vec<VEC>(cp + (int64_t)q1 * P.ld_in);
            if (q2 < k) u2 = load_vec<VEC>(cp + (int64_t)q2 * P.ld_in);
            if (q3 < k) u3 = load_vec<VEC>(cp + (int64_t)q3 * P.ld_in);
            store_vec<VEC>(bp + row * L.stride, u0);
            if (q1 < k) store_vec<VEC>(bp + q1 * L.stride, u1);
            if (q2 < k) store_vec<VEC>(bp + q2 * L.stride, u2);
            if (q3 < k) store_vec<VEC>(bp + q3 * L.stride, u3);
        }
    }
}

// ---------------------------------------------------------------------------------------
// row gather-FMA from LDS and store
// ---------------------------------------------------------------------------------------
template <int S, int VEC>
__device__ __forceinline__ void compute_staged(const LaunchParams& P, const WorkItem& it,
                                               const int* sm, int lane)
{
    using V = Vec<VEC>;
    const StagedLayout L = staged_layout(it.m, it.k, it.nnz, it.fw, P.pad);
    const int2* cv = reinterpret_cast<const int2*>(sm + L.cv_off);
    const float* bs = reinterpret_cast<const float*>(sm + L.b_off);
    const Split<S, VEC> sp(it.fw, lane);
    float* __restrict__ dst = P.out + it.out_row_off * P.ld_out + it.f0;

    const int row_end = it.row0 + it.nrows;
    for (int r = it.row0 + sp.g; r < row_end; r += sp.groups) {
        const int p0 = sm[r];
        const int p1 = sm[r + 1];
        for (int v = sp.l; v < sp.nvec; v += sp.g_lanes) {
            const float* bcol = bs + v * VEC;
            typename V::type acc = V::zero();
            int p = p0;
            for (; p + 3 < p1; p += 4) {
                const int2 e0 = cv[p], e1 = cv[p + 1], e2 = cv[p + 2], e3 = cv[p + 3];
                const typename V::type b0 = load_vec<VEC>(bcol + e0.x * L.stride);
                const typename V::type b1 = load_vec<VEC>(bcol + e1.x * L.stride);
                const typename V::type b2 = load_vec<VEC>(bcol + e2.x * L.stride);
                const typename V::type b3 = load_vec<VEC>(bcol + e3.x * L.stride);
                V::fma(acc, __int_as_float(e0.y), b0);
                V::fma(acc, __int_as_float(e1.y), b1);
                V::fma(acc, __int_as_float(e2.y), b2);
                V::fma(acc, __int_as_float(e3.y), b3);
            }
            for (; p < p1; ++p) {
                const int2 e = cv[p];
                V::fma(acc, __int_as_float(e.y), load_vec<VEC>(bcol + e.x * L.stride));
            }
            store_vec<VEC>(dst + (int64_t)r * P.ld_out + v * VEC, acc);
        }
    }
}

// Generic bin: nothing staged, every operand comes from global memory (L2 keeps the dense
// block of a large operation while its row blocks run on the same XCD).
template <int VEC>
__device__ __forceinline__ void compute_generic(const LaunchParams& P, const WorkItem& it,
                                                int lane)
{
    using V = Vec<VEC>;
    const Split<kThreads, VEC> sp(it.fw, lane);
    const int32_t* __restrict__ rp = P.rpt + it.rpt_off;
    const int32_t* __restrict__ ci = P.colids + it.nz_off;
    const float* __restrict__ va = P.values + it.nz_off;
    const float* __restrict__ src = P.in + it.in_row_off * P.ld_in + it.f0;
    float* __restrict__ dst = P.out + it.out_row_off * P.ld_out + it.f0;

    for (int r = it.row0 + sp.g; r < it.row0 + it.nrows; r += sp.groups) {
        const int p0 = rp[r];
        const int p1 = rp[r + 1];
        for (int v = sp.l; v < sp.nvec; v += sp.g_lanes) {
            const float* bcol = src + v * VEC;
            typename V::type acc = V::zero();
            int p = p0;
            for (; p + 3 < p1; p += 4) {
                const int c0 = ci[p], c1 = ci[p + 1], c2 = ci[p + 2], c3 = ci[p + 3];
                const float a0 = va[p], a1 = va[p + 1], a2 = va[p + 2], a3 = va[p + 3];
                const typename V::type b0 = load_vec<VEC>(bcol + (int64_t)c0 * P.ld_in);
                const typename V::type b1 = load_vec<VEC>(bcol + (int64_t)c1 * P.ld_in);
                const typename V::type b2 = load_vec<VEC>(bcol + (int64_t)c2 * P.ld_in);
                const typename V::type b3 = load_vec<VEC>(bcol + (int64_t)c3 * P.ld_in);
                V::fma(acc, a0, b0);
                V::fma(acc, a1, b1);
                V::fma(acc, a2, b2);
                V::fma(acc, a3, b3);
            }
            for (; p < p1; ++p)
                V::fma(acc, va[p], load_vec<VEC>(bcol + (int64_t)ci[p] * P.ld_in));
            store_vec<VEC>(dst + (int64_t)r * P.ld_out + v * VEC, acc);
        }
    }
}

// A workgroup of a sub-workgroup range: 256/S slots, one staged item each.
template <int LOG2S, int VEC>
__device__ __forceinline__ void run_slots(const LaunchParams& P, int* sm, int range, int wrel)
{
    constexpr int S = 1 << LOG2S;
    constexpr int SLOTS = kThreads / S;
    const int tid = threadIdx.x;
    const int slot = tid >> LOG2S;
    const int lane = tid & (S - 1);
    int idx = P.item_base[range] + wrel * SLOTS + slot;
    if (LOG2S == 6) idx = __builtin_amdgcn_readfirstlane(idx);   // uniform inside a wavefront
    const WorkItem it = P.items[idx];
    int* slot_sm = sm + slot * (P.lds_floats >> (8 - LOG2S));
    if (it.nrows > 0) stage_item<S, VEC>(P, it, slot_sm, lane);
    __syncthreads();
    if (it.nrows > 0) compute_staged<S, VEC>(P, it, slot_sm, lane);
}

#ifdef BSPMM_TRACE
#define BSPMM_STAMP(slot)                                                              \
    do {                                                                               \
        if (P.trace) {                                                                 \
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");                \
            if (threadIdx.x == 0) P.trace[(size_t)blockIdx.x * 8 + (slot)] = wall_clock64(); \
        }                                                                              \
    } while (0)
#else
#define BSPMM_STAMP(slot) do { } while (0)
#endif

template <int VEC>
__global__ void __launch_bounds__(kThreads) bspmm_kernel(const LaunchParams P)
{
    extern __shared__ __align__(16) int sm[];
    const int w = blockIdx.x;
#ifdef BSPMM_TRACE
    if (P.trace && threadIdx.x == 0) P.trace[(size_t)blockIdx.x * 8] = wall_clock64();
#endif
    if (w < P.wg_end[0]) {
        const WorkItem it = P.items[P.item_base[0] + w];   // uniform address: scalar loads
        if (it.nrows <= 0) return;
        BSPMM_STAMP(1);
        if (it.staged) {
            stage_item<kThreads, VEC>(P, it, sm, threadIdx.x);
            __syncthreads();
            BSPMM_STAMP(2);
            compute_staged<kThreads, VEC>(P, it, sm, threadIdx.x);
        } else {
            compute_generic<VEC>(P, it, threadIdx.x);
        }
        BSPMM_STAMP(3);
#ifdef BSPMM_TRACE
        if (P.trace && threadIdx.x == 0) {
            P.trace[(size_t)blockIdx.x * 8 + 4] = it.nrows;
            P.trace[(size_t)blockIdx.x * 8 + 5] = it.k;
            P.trace[(size_t)blockIdx.x * 8 + 6] = it.nnz;
            unsigned hw;
            asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(hw));
            P.trace[(size_t)blockIdx.x * 8 + 7] = hw;
        }
#endif
    } else if (w < P.wg_end[1]) {
        run_slots<6, VEC>(P, sm, 1, w - P.wg_end[0]);
    } else if (w < P.wg_end[2]) {
        run_slots<5, VEC>(P, sm, 2, w - P.wg_end[1]);
    } else {
        run_slots<4, VEC>(P, sm, 3, w - P.wg_end[2]);
    }
}

// ---------------------------------------------------------------------------------------
// transposed CSR build: one workgroup per operation.
//   count entries per column -> exclusive prefix sum (row pointers of A^T) -> scatter the
//   entry positions with atomic cursors (arrival order is arbitrary) -> every entry finds its
//   rank inside its column segment by counting the positions smaller than its own.
// The result does not depend on the arrival order: it is the stable transpose.
// `work` is k+1 counters followed by nnz positions, in LDS when it fits, else in global
// scratch (both reached through flat addressing).
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kThreads)
build_transpose_kernel(const OpRecord* __restrict__ ops, const int32_t* __restrict__ rpt,
                       const int32_t* __restrict__ colids, const float* __restrict__ values,
                       int32_t* __restrict__ rpt_t, int32_t* __restrict__ colids_t,
                       float* __restrict__ values_t, int32_t* gscratch)
{
    extern __shared__ __align__(16) int sm[];
    __shared__ int partial[kThreads];
    const OpRecord o = ops[blockIdx.x];
    const int tid = threadIdx.x;
    const int k = o.k, m = o.m, nnz = o.nnz;
    int* cnt = o.scratch_off >= 0 ? gscratch + o.scratch_off : sm;   // k+1 ints
    int* pos = cnt + (k + 1);                                          // nnz ints
    const int32_t* ci = colids + o.nz_off;
    const int32_t* rp = rpt + o.rpt_off;
    int32_t* rt = rpt_t + o.rpt_t_off;

    for (int c = tid; c <= k; c += kThreads) cnt[c] = 0;
    __syncthreads();
    for (int p = tid; p < nnz; p += kThreads) {
        const int c = ci[p];
        if ((unsigned)c < (unsigned)k) atomicAdd(&cnt[c + 1], 1);
    }
    __syncthreads();

    // inclusive scan of cnt[0..k]: afterwards cnt[c] = first position of column c
    const int chunk = (k + 1 + kThreads - 1) / kThreads;
    const int lo = tid * chunk;
    const int hi = lo + chunk < k + 1 ? lo + chunk : k + 1;
    int sum = 0;
    for (int c = lo; c < hi; ++c) sum += cnt[c];
    partial[tid] = sum;
    __syncthreads();
    for (int d = 1; d < kThreads; d <<= 1) {
        const int add = tid >= d ? partial[tid - d] : 0;
        __syncthreads();
        partial[tid] += add;
        __syncthreads();
    }
    int run = tid > 0 ? partial[tid - 1] : 0;
    for (int c = lo; c < hi; ++c) {
        run += cnt[c];
        cnt[c] = run;
        rt[c] = run;
    }
    __syncthreads();

    // scatter positions; cnt[c] ends as the first position of column c+1
    for (int p = tid; p < nnz; p += kThreads) {
        const int c = ci[p];
        if ((unsigned)c < (unsigned)k) pos[atomicAdd(&cnt[c], 1)] = p;
    }
    __syncthreads();

    const float* va = values + o.nz_off;
    for (int q = tid; q < nnz; q += kThreads) {
        const int p = pos[q];
        const int c = ci[p];
        const int beg = c > 0 ? cnt[c - 1] : 0;
        const int end = cnt[c];
        int rank = 0;
        for (int t = beg; t < end; ++t) rank += pos[t] < p ? 1 : 0;
        // row of entry p: the last r with rp[r] <= p
        int a = 0, b = m;   // invariant: rp[a] <= p, and (b == m or rp[b] > p) ... search (a, b]
        while (b - a > 1) {
            const int mid = (a + b) >> 1;
            if (rp[mid] <= p) a = mid; else b = mid;
        }
        colids_t[o.nz_t_off + beg + rank] = a;
        values_t[o.nz_t_off + beg + rank] = va[p];
    }
}

// ---------------------------------------------------------------------------------------
// structural check: *flag becomes the smallest index of a malformed operation.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kThreads)
validate_csr_kernel(const OpRecord* __restrict__ ops, const int32_t* __restrict__ rpt,
                    const int32_t* __restrict__ colids, int32_t* flag)
{
    const OpRecord o = ops[blockIdx.x];
    const int tid = threadIdx.x;
    bool bad = false;
    if (o.m > 0) {
        const int32_t* rp = rpt + o.rpt_off;
        if (tid == 0 && (rp[0] != 0 || rp[o.m] != o.nnz)) bad = true;
        for (int r = tid; r < o.m; r += kThreads)
            if (rp[r + 1] < rp[r]) bad = true;
    } else if (o.nnz != 0) {
        bad = true;
    }
    const int32_t* ci = colids + o.nz_off;
    for (int p = tid; p < o.nnz; p += kThreads)
        if ((unsigned)ci[p] >= (unsigned)o.k) bad = true;
    if (bad) atomicMin(flag, (int)blockIdx.x);
}

__global__ void fill_i32_kernel(int32_t* p, int32_t v, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// ---------------------------------------------------------------------------------------
// host-side launchers (the only symbols the rest of the library sees)
// ---------------------------------------------------------------------------------------
hipError_t launch_bspmm(const LaunchParams& P, int grid, int lds_bytes, bool vec4,
                        hipStream_t stream)
{
    if (grid <= 0) return hipSuccess;
    if (vec4)
        hipLaunchKernelGGL(bspmm_kernel<4>, dim3(grid), dim3(kThreads), lds_bytes, stream, P);
    else
        hipLaunchKernelGGL(bspmm_kernel<1>, dim3(grid), dim3(kThreads), lds_bytes, stream, P);
    return hipGetLastError();
}

hipError_t launch_build_transpose(const OpRecord* ops, int batch, int lds_bytes,
                                  const int32_t* rpt, const int32_t* colids,
                                  const float* values, int32_t* rpt_t, int32_t* colids_t,
                                  float* values_t, int32_t* gscratch, hipStream_t stream)
{
    if (batch <= 0) return hipSuccess;
    hipLaunchKernelGGL(build_transpose_kernel, dim3(batch), dim3(kThreads), lds_bytes, stream,
                       ops, rpt, colids, values, rpt_t, colids_t, values_t, gscratch);
    return hipGetLastError();
}

hipError_t launch_validate(const OpRecord* ops, int batch, const int32_t* rpt,
                           const int32_t* colids, int32_t* flag, hipStream_t stream)
{
    hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(64), 0, stream, flag, 0x7fffffff, 1);
    if (batch > 0)
        hipLaunchKernelGGL(validate_csr_kernel, dim3(batch), dim3(kThreads), 0, stream, ops, rpt,
                           colids, flag);
    return hipGetLastError();
}

}  // namespace bspmm
