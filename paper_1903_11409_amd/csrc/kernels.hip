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
// staging: global -> LDS.  All three copies are independent of each other, so their loads
// are in flight together; nothing here depends on the contents of the CSR arrays.
// ---------------------------------------------------------------------------------------
template <int S, int VEC>
__device__ __forceinline__ void stage_item(const LaunchParams& P, const WorkItem& it, int* sm,
                                           int lane)
{
    const StagedLayout L = staged_layout(it.m, it.k, it.nnz, it.fw, P.pad);

    const int32_t* __restrict__ rp = P.rpt + it.rpt_off;
    for (int i = lane; i <= it.m; i += S) {
        int v = rp[i];
        v = v < 0 ? 0 : v;
        sm[i] = v > it.nnz ? it.nnz : v;   // a malformed row pointer cannot leave the slot
    }

    const int32_t* __restrict__ ci = P.colids + it.nz_off;
    const float* __restrict__ va = P.values + it.nz_off;
    int2* cv = reinterpret_cast<int2*>(sm + L.cv_off);
    for (int p = lane; p < it.nnz; p += S) {
        int c = ci[p];
        c = (unsigned)c < (unsigned)it.k ? c : 0;   // a malformed column cannot leave the tile
        cv[p] = make_int2(c, __float_as_int(va[p]));
    }

    const Split<S, VEC> sp(it.fw, lane);
    float* bs = reinterpret_cast<float*>(sm + L.b_off);
    const float* __restrict__ src = P.in + it.in_row_off * P.ld_in + it.f0;
    for (int v = sp.l; v < sp.nvec; v += sp.g_lanes) {
        const int step = sp.groups;
        int row = sp.g;
        // four rows per trip so that four loads are outstanding before the first LDS write
        for (; row + 3 * step < it.k; row += 4 * step) {
            typename Vec<VEC>::type t0 = load_vec<VEC>(src + (int64_t)(row) * P.ld_in + v * VEC);
            typename Vec<VEC>::type t1 = load_vec<VEC>(src + (int64_t)(row + step) * P.ld_in + v * VEC);
            typename Vec<VEC>::type t2 = load_vec<VEC>(src + (int64_t)(row + 2 * step) * P.ld_in + v * VEC);
            typename Vec<VEC>::type t3 = load_vec<VEC>(src + (int64_t)(row + 3 * step) * P.ld_in + v * VEC);
            store_vec<VEC>(bs + (row) * L.stride + v * VEC, t0);
            store_vec<VEC>(bs + (row + step) * L.stride + v * VEC, t1);
            store_vec<VEC>(bs + (row + 2 * step) * L.stride + v * VEC, t2);
            store_vec<VEC>(bs + (row + 3 * step) * L.stride + v * VEC, t3);
        }
        for (; row < it.k; row += step)
            store_vec<VEC>(bs + row * L.stride + v * VEC,
                           load_vec<VEC>(src + (int64_t)row * P.ld_in + v * VEC));
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

    for (int r = sp.g; r < it.nrows; r += sp.groups) {
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

template <int VEC>
__global__ void __launch_bounds__(kThreads) bspmm_kernel(const LaunchParams P)
{
    extern __shared__ __align__(16) int sm[];
    const int w = blockIdx.x;
    if (w < P.wg_end[0]) {
        const WorkItem it = P.items[P.item_base[0] + w];   // uniform address: scalar loads
        if (it.nrows <= 0) return;
        if (it.staged) {
            stage_item<kThreads, VEC>(P, it, sm, threadIdx.x);
            __syncthreads();
            compute_staged<kThreads, VEC>(P, it, sm, threadIdx.x);
        } else {
            compute_generic<VEC>(P, it, threadIdx.x);
        }
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
