// Device kernels of libbspmm for gfx950 (wave64).
//
// bspmm_kernel      one launch computes every work item of a schedule: per item, stage the
//                   operation's CSR arrays and the feature tile of its dense input in LDS
//                   (or, for the generic bin, read them from global memory), then give every
//                   output row a group of lanes that accumulates its stored entries in
//                   registers and writes the row once (the row-wise, atomic-free product of
//                   Fig. 4, batched as in Sec. IV-C, with the column blocking of Fig. 5(d)).
// bspmm_lean_kernel the same product for launches made only of whole-workgroup items on the
//                   float4 path: items carry what the general kernel derives, the dense tile
//                   goes global -> LDS directly.
// bspmm_gcn_kernel  the fused front of the graph-convolution layer (Fig. 7): the dense tile is
//                   made on the matrix cores from the layer input and the weights, for one
//                   channel or for all channels of the layer, and gathered as above.
// bspmm_gcn_stream_kernel  the same layer for large batches: resident workgroups with the
//                   weights in registers stream the graphs of host-made lists through LDS.
// bspmm_coo_kernel  the direct product for COO / SparseTensor operands (Fig. 3, Fig. 5(a,b)).
// build_sorted      stable CSR -> transposed CSR of every operation (counting sort by column),
//                   and COO / SparseTensor -> CSR (the same sort by row).
// merge_sets        merged CSR of operations that are summed into one output block.
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

// Output rows are written once and never read by this launch: a non-temporal store keeps
// them from displacing the dense blocks that the generic bin re-reads out of L2.
template <int VEC>
__device__ __forceinline__ void store_out(float* p, const typename Vec<VEC>::type& v)
{
    if constexpr (VEC == 4) {
        typedef float native4 __attribute__((ext_vector_type(4)));
        native4 n = {v.x, v.y, v.z, v.w};
        __builtin_nontemporal_store(n, reinterpret_cast<native4*>(p));
    } else {
        __builtin_nontemporal_store(v, p);
    }
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
// (the pointer travels in the slot of the front's weights, which such launches do not have: a
// field of its own made the argument block longer and the headline launch 1 % slower)
__device__ __forceinline__ const int32_t* merged_words(const LaunchParams& P)
{
    return reinterpret_cast<const int32_t*>(P.w);
}

template <int S, int VEC, bool HUBS, bool WITH_TILE = true, bool MERGED = false>
__device__ __forceinline__ void stage_item(const LaunchParams& P, const WorkItem& it, int* sm,
                                           int lane)
{
    using VT = typename Vec<VEC>::type;
    const StagedLayout L = staged_layout(it.m, it.k, it.nnz, it.fw, P.pad, HUBS && S == kThreads);
    if (HUBS && S == kThreads && lane == 0) sm[L.hub_off] = 0;   // no hub row found yet
    // (MERGED kernels, bit 2 of `staged`: the item is a set of summed operations that read one
    // dense block, i.e. the product with the sum of their matrices; its CSR is the set's
    // merged one in the workspace - row pointers at rpt_off, columns at nz_off, values behind
    // the columns.  A template parameter, not a run-time test alone: the three selects cost
    // the plain kernel 2 % of the headline launch.)
    const bool merged = MERGED && (it.staged & 4) != 0;
    const int32_t* __restrict__ rp = (merged ? merged_words(P) : P.rpt) + it.rpt_off;
    const int32_t* __restrict__ ci = (merged ? merged_words(P) : P.colids) + it.nz_off;
    const float* __restrict__ va =
        merged ? reinterpret_cast<const float*>(merged_words(P) + it.nz_off + round_up(it.nnz, 4))
               : P.values + it.nz_off;
    int2* cv = reinterpret_cast<int2*>(sm + L.cv_off);
    float* bs = reinterpret_cast<float*>(sm + L.b_off);
    const float* __restrict__ src = P.in + it.in_row_off * P.ld_in + it.f0;
    const Split<S, VEC> sp(it.fw, lane);
    const int step = sp.groups;
    const int m = it.m, nnz = it.nnz, k = it.k;

    // ---- first trip of every copy: loads only
    // (unconditional, from a clamped index: a load inside a branch drags the first use of its
    // value, and with it a wait for the whole round trip, in front of the loads that follow)
    const int rv = rp[min(lane, m)];
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
    // Dense tile.  Fast path: when a tile row is a power-of-two number of float4 and rows are
    // packed without padding, whole wavefronts copy 1 KiB at a time straight from global
    // memory into LDS (lane i lands at base + 16*i): no staging registers, and the entire
    // tile is in flight at once instead of four rows per lane group.
    const bool direct = WITH_TILE && VEC == 4 && S >= 64 && P.pad == 0 && (sp.nvec & (sp.nvec - 1)) == 0;
    if (direct) {
        const int sh = ilog2(sp.nvec);
        const int total = k << sh;                       // float4 in the tile
        const int wl = lane & 63;
        for (int e0 = (lane >> 6) << 6; e0 < total; e0 += S) {
            const int e = e0 + wl;
            if (e < total) {
                const float* gp = src + (int64_t)(e >> sh) * P.ld_in + ((e & (sp.nvec - 1)) << 2);
                // a dense tile that no other item reads is streamed (non-temporal) so that it
                // does not displace data other workgroups re-read from L2
                if (it.staged & 2)
                    __builtin_amdgcn_global_load_lds(
                        (const void __attribute__((address_space(1)))*)gp,
                        (void __attribute__((address_space(3)))*)(bs + (e0 << 2)), 16, 0, 2);
                else
                    __builtin_amdgcn_global_load_lds(
                        (const void __attribute__((address_space(1)))*)gp,
                        (void __attribute__((address_space(3)))*)(bs + (e0 << 2)), 16, 0, 0);
            }
        }
    }
    const bool col_ok = WITH_TILE && !direct && sp.l < sp.nvec;
    const int r0 = sp.g, r1 = sp.g + step, r2 = sp.g + 2 * step, r3 = sp.g + 3 * step;
    const float* colp = src + sp.l * VEC;
    VT t0 = Vec<VEC>::zero(), t1 = Vec<VEC>::zero(), t2 = Vec<VEC>::zero(), t3 = Vec<VEC>::zero();
    if (WITH_TILE && !direct) {     // the same for every lane: a scalar branch over the whole path
        if (col_ok && r0 < k) t0 = load_vec<VEC>(colp + (int64_t)r0 * P.ld_in);
        if (col_ok && r1 < k) t1 = load_vec<VEC>(colp + (int64_t)r1 * P.ld_in);
        if (col_ok && r2 < k) t2 = load_vec<VEC>(colp + (int64_t)r2 * P.ld_in);
        if (col_ok && r3 < k) t3 = load_vec<VEC>(colp + (int64_t)r3 * P.ld_in);
    }

    // No use of a loaded value may be scheduled above this line: the wait in front of it would
    // hold back the loads that have not been issued yet and cost a second round trip.
    __builtin_amdgcn_sched_barrier(0);

    // ---- first trip: LDS writes.  Row pointers are clamped to [0, nnz] and columns to
    // [0, k) so that malformed arrays cannot make a lane leave its slot.
    if (lane <= m) sm[lane] = min(max(rv, 0), nnz);
    // (entries carry the word offset of their dense row in the tile, not the column itself:
    // the multiplication is done once here instead of by every lane that gathers the entry)
    if (lane < nnz)
        cv[lane] = make_int2((unsigned)c0 < (unsigned)k ? c0 * L.stride : 0, __float_as_int(a0));
    if (lane + S < nnz)
        cv[lane + S] = make_int2((unsigned)c1 < (unsigned)k ? c1 * L.stride : 0, __float_as_int(a1));
    float* bcol = bs + sp.l * VEC;
    if (WITH_TILE && !direct) {
        if (col_ok && r0 < k) store_vec<VEC>(bcol + r0 * L.stride, t0);
        if (col_ok && r1 < k) store_vec<VEC>(bcol + r1 * L.stride, t1);
        if (col_ok && r2 < k) store_vec<VEC>(bcol + r2 * L.stride, t2);
        if (col_ok && r3 < k) store_vec<VEC>(bcol + r3 * L.stride, t3);
    }

    // ---- leftovers of larger items (each behind a condition that is the same for every
    // lane, so that a small item jumps over them instead of walking through masked-off code)
    if (m >= S)
        for (int i = lane + S; i <= m; i += S) sm[i] = min(max(rp[i], 0), nnz);
    if (nnz > 2 * S)
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
        cv[p] = make_int2((unsigned)cc0 < (unsigned)k ? cc0 * L.stride : 0, __float_as_int(aa0));
        if (q < nnz)
            cv[q] = make_int2((unsigned)cc1 < (unsigned)k ? cc1 * L.stride : 0, __float_as_int(aa1));
    }
    if (WITH_TILE && !direct)
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
// split-row reduce.  A hub row (hundreds of entries) would keep one lane group busy long after
// the rest of the workgroup has finished, so its entries are dealt out to ALL lane groups of
// the workgroup; each lane then holds a partial sum for its columns, and the partial sums of the
// groups are added up: inside a wavefront with DPP row rotations (distance < 16),
// ds_swizzle (16) and ds_bpermute (32), across the four wavefronts through one tile row of LDS
// each, in a fixed order (the result does not depend on timing).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float add_from_lane_xor(float v, int off)
{
    switch (off) {
        case 1: return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x121, 0xf, 0xf, false));
        case 2: return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x122, 0xf, 0xf, false));
        case 4: return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x124, 0xf, 0xf, false));
        case 8: return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x128, 0xf, 0xf, false));
        case 16: return v + __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(v), (16 << 10) | 0x1f));
        default: return v + __shfl_xor(v, 32);
    }
}

// Sum over the lane groups of one wavefront: afterwards every lane holds the total of the
// lanes that share its position inside a group (rotations by g, 2g, ... inside rows of 16
// lanes visit every group of the row; 16 and 32 are true exchanges).
template <int VEC>
__device__ __forceinline__ void wave_group_sum(typename Vec<VEC>::type& a, int g_lanes)
{
    for (int off = g_lanes; off < 64; off <<= 1) {
        if constexpr (VEC == 4) {
            a.x = add_from_lane_xor(a.x, off);
            a.y = add_from_lane_xor(a.y, off);
            a.z = add_from_lane_xor(a.z, off);
            a.w = add_from_lane_xor(a.w, off);
        } else {
            a = add_from_lane_xor(a, off);
        }
    }
}

// One hub row computed by the whole workgroup.  `load_entry(p)` yields (column, value) of entry
// p, `bcol` addresses this lane's vector of dense row 0, `stride` is the dense row stride.
// Contains two barriers: every lane of the workgroup must call it.
template <int VEC, typename Entry>
__device__ __forceinline__ void hub_row(int p0, int p1, Entry load_entry, const float* bcol,
                                        int64_t stride, bool col_ok, int g_lanes, int groups,
                                        int g, int l, float* scratch, int fwp, float* out_row)
{
    using V = Vec<VEC>;
    using VT = typename V::type;
    VT acc = V::zero();
    if (col_ok) {
        int p = p0 + g;
        for (; p + 3 * groups < p1; p += 4 * groups) {
            const int2 e0 = load_entry(p), e1 = load_entry(p + groups),
                       e2 = load_entry(p + 2 * groups), e3 = load_entry(p + 3 * groups);
            const VT b0 = load_vec<VEC>(bcol + e0.x * stride);
            const VT b1 = load_vec<VEC>(bcol + e1.x * stride);
            const VT b2 = load_vec<VEC>(bcol + e2.x * stride);
            const VT b3 = load_vec<VEC>(bcol + e3.x * stride);
            V::fma(acc, __int_as_float(e0.y), b0);
            V::fma(acc, __int_as_float(e1.y), b1);
            V::fma(acc, __int_as_float(e2.y), b2);
            V::fma(acc, __int_as_float(e3.y), b3);
        }
        for (; p < p1; p += groups) {
            const int2 e = load_entry(p);
            V::fma(acc, __int_as_float(e.y), load_vec<VEC>(bcol + e.x * stride));
        }
    }
    wave_group_sum<VEC>(acc, g_lanes);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) < g_lanes && col_ok) store_vec<VEC>(scratch + wave * fwp + l * VEC, acc);
    __syncthreads();
    if (threadIdx.x < g_lanes && col_ok) {
        VT t = load_vec<VEC>(scratch + l * VEC);
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) {
            const VT u = load_vec<VEC>(scratch + w * fwp + l * VEC);
            if constexpr (VEC == 4) {
                t.x += u.x; t.y += u.y; t.z += u.z; t.w += u.w;
            } else {
                t += u;
            }
        }
        store_out<VEC>(out_row + l * VEC, t);
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------------------
// row gather-FMA from LDS and store
// ---------------------------------------------------------------------------------------
// `tile_shift` moves the dense tile behind a guest that sits at its usual place (the layer
// input of the fused front); ACC adds the sums to the output instead of overwriting it.
template <int S, int VEC, bool HUBS, bool ACC = false>
__device__ __forceinline__ void compute_staged(const LaunchParams& P, const WorkItem& it,
                                               int* sm, int lane, int tile_shift = 0)
{
    using V = Vec<VEC>;
    constexpr bool kHubs = HUBS && S == kThreads;
    const StagedLayout L = staged_layout(it.m, it.k, it.nnz, it.fw, P.pad, kHubs);
    const int2* cv = reinterpret_cast<const int2*>(sm + L.cv_off);
    const float* bs = reinterpret_cast<const float*>(sm + L.b_off + tile_shift);
    const Split<S, VEC> sp(it.fw, lane);
    float* __restrict__ dst = P.out + it.out_row_off * P.ld_out + it.f0;
    // hub rows need one vector per lane (always true on the float4 path)
    const bool hubs_on = kHubs && sp.nvec <= sp.g_lanes;
    const int hub_deg = max(kHubMin, kHubRatio * ((it.nnz + it.m - 1) / max(it.m, 1)));
    int* hub = sm + L.hub_off;

    const int row_end = it.row0 + it.nrows;
    for (int r = it.row0 + sp.g; r < row_end; r += sp.groups) {
        const int p0 = sm[r];
        const int p1 = sm[r + 1];
        if (hubs_on && p1 - p0 >= hub_deg) {
            // left to the whole workgroup.  The list has room for nnz / kHubMin rows, which is
            // all there can be when the row pointers are monotone; malformed ones (clamped, but
            // going up and down) could name more: those rows stay out of the list, and so
            // inside the item's LDS (their output is not written; the arrays were malformed).
            if (sp.l == 0) {
                const int slot = atomicAdd(&hub[0], 1);
                if (slot < it.nnz / kHubMin) hub[1 + slot] = r;
            }
            continue;
        }
        for (int v = sp.l; v < sp.nvec; v += sp.g_lanes) {
            const float* bcol = bs + v * VEC;
            typename V::type acc = V::zero();
            int p = p0;
            for (; p + 3 < p1; p += 4) {
                const int2 e0 = cv[p], e1 = cv[p + 1], e2 = cv[p + 2], e3 = cv[p + 3];
                const typename V::type b0 = load_vec<VEC>(bcol + e0.x);
                const typename V::type b1 = load_vec<VEC>(bcol + e1.x);
                const typename V::type b2 = load_vec<VEC>(bcol + e2.x);
                const typename V::type b3 = load_vec<VEC>(bcol + e3.x);
                V::fma(acc, __int_as_float(e0.y), b0);
                V::fma(acc, __int_as_float(e1.y), b1);
                V::fma(acc, __int_as_float(e2.y), b2);
                V::fma(acc, __int_as_float(e3.y), b3);
            }
            for (; p < p1; ++p) {
                const int2 e = cv[p];
                V::fma(acc, __int_as_float(e.y), load_vec<VEC>(bcol + e.x));
            }
            if constexpr (ACC) {
                static_assert(VEC == 4, "accumulating stores are built for the float4 path");
                const float4 old = load_vec<4>(dst + (int64_t)r * P.ld_out + v * VEC);
                acc.x += old.x;
                acc.y += old.y;
                acc.z += old.z;
                acc.w += old.w;
            }
            store_out<VEC>(dst + (int64_t)r * P.ld_out + v * VEC, acc);
        }
    }
    if constexpr (kHubs) {
        if (!hubs_on) return;          // uniform: depends on the item only
        __syncthreads();               // the hub list is complete
        const int n_hub = min(hub[0], it.nnz / kHubMin);
        const int fwp = round_up(it.fw, 4);
        float* scratch = reinterpret_cast<float*>(hub + round_up(1 + it.nnz / kHubMin, 4));
        for (int h = 0; h < n_hub; ++h) {
            const int r = hub[1 + h];
            hub_row<VEC>(sm[r], sm[r + 1], [cv](int p) { return cv[p]; }, bs + sp.l * VEC,
                         (int64_t)1 /* entries hold row offsets already */, sp.l < sp.nvec, sp.g_lanes, sp.groups, sp.g, sp.l,
                         scratch, fwp, dst + (int64_t)r * P.ld_out);
        }
    }
}

// Generic bin: the operation's dense tile does not fit LDS, so a row block gathers it from
// global memory (L2 keeps the block while the row blocks of one operation run on one XCD).
// Only the block's slice of the CSR arrays is staged, in two dependent steps (row pointers,
// then the entries they delimit); after that every gather of a row is independent and up to
// four are in flight per lane (deeper
// unrolling costs registers, hence occupancy, and measured slower).
template <int VEC, bool HUBS>
__device__ __forceinline__ void run_generic(const LaunchParams& P, const WorkItem& it, int* sm,
                                            int tid)
{
    using V = Vec<VEC>;
    using VT = typename V::type;
    const int32_t* __restrict__ rp = P.rpt + it.rpt_off + it.row0;
    const int32_t* __restrict__ ci = P.colids + it.nz_off;
    const float* __restrict__ va = P.values + it.nz_off;
    const int nrows = it.nrows;
    for (int i = tid; i <= nrows; i += kThreads) sm[i] = min(max(rp[i], 0), it.nnz);
    __syncthreads();
    const int pbeg = __builtin_amdgcn_readfirstlane(sm[0]);
    const int cnt = max(__builtin_amdgcn_readfirstlane(sm[nrows]) - pbeg, 0);
    const int cv_off = round_up(nrows + 1, 2);
    const int hub_off = round_up(cv_off + 2 * cnt, 4);
    const bool fits = hub_off + (HUBS ? hub_words(nrows, it.fw) : 0) <= P.lds_floats;
    int2* cv = reinterpret_cast<int2*>(sm + cv_off);
    int* hub = sm + hub_off;
    if (fits) {
        if (HUBS && tid == 0) hub[0] = 0;
        for (int p = tid; p < cnt; p += 2 * kThreads) {
            const int q = p + kThreads;
            const int c0 = ci[pbeg + p];
            const float a0 = va[pbeg + p];
            int c1 = 0;
            float a1 = 0.f;
            if (q < cnt) {
                c1 = ci[pbeg + q];
                a1 = va[pbeg + q];
            }
            cv[p] = make_int2((unsigned)c0 < (unsigned)it.k ? c0 : 0, __float_as_int(a0));
            if (q < cnt) cv[q] = make_int2((unsigned)c1 < (unsigned)it.k ? c1 : 0, __float_as_int(a1));
        }
    }
    __syncthreads();

    const Split<kThreads, VEC> sp(it.fw, tid);
    const float* __restrict__ src = P.in + it.in_row_off * P.ld_in + it.f0;
    float* __restrict__ dst = P.out + (it.out_row_off + it.row0) * P.ld_out + it.f0;
    const bool hubs_on = HUBS && fits && sp.nvec <= sp.g_lanes;
    const int hub_deg = HUBS ? max(kHubMin, kHubRatio * ((it.nnz + it.m - 1) / max(it.m, 1))) : 0;
    for (int i = sp.g; i < nrows; i += sp.groups) {
        const int p0 = sm[i] - pbeg;
        const int p1 = sm[i + 1] - pbeg;
        if (hubs_on && p1 - p0 >= hub_deg) {
            if (sp.l == 0) hub[1 + atomicAdd(&hub[0], 1)] = i;   // left to the whole workgroup
            continue;
        }
        for (int v = sp.l; v < sp.nvec; v += sp.g_lanes) {
            const float* bcol = src + v * VEC;
            VT acc = V::zero();
            for (int p = p0; p < p1; p += 4) {
                int cc[4];
                float aa[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int q = min(p + u, p1 - 1);
                    if (fits) {
                        const int2 e = cv[q];
                        cc[u] = e.x;
                        aa[u] = __int_as_float(e.y);
                    } else {
                        const int c = ci[pbeg + q];
                        cc[u] = (unsigned)c < (unsigned)it.k ? c : 0;
                        aa[u] = va[pbeg + q];
                    }
                    if (p + u >= p1) aa[u] = 0.f;
                }
                VT b[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    b[u] = V::zero();
                    if (p + u < p1) b[u] = load_vec<VEC>(bcol + (int64_t)cc[u] * P.ld_in);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) V::fma(acc, aa[u], b[u]);
            }
            store_out<VEC>(dst + (int64_t)i * P.ld_out + v * VEC, acc);
        }
    }
    if (!HUBS || !hubs_on) return;     // uniform: depends on the item and its row pointers
    __syncthreads();                   // the hub list is complete
    const int n_hub = hub[0];
    const int fwp = round_up(it.fw, 4);
    float* scratch = reinterpret_cast<float*>(hub + round_up(1 + nrows, 4));
    for (int h = 0; h < n_hub; ++h) {
        const int i = hub[1 + h];
        hub_row<VEC>(sm[i] - pbeg, sm[i + 1] - pbeg, [cv](int p) { return cv[p]; },
                     src + sp.l * VEC, P.ld_in, sp.l < sp.nvec, sp.g_lanes, sp.groups, sp.g, sp.l,
                     scratch, fwp, dst + (int64_t)i * P.ld_out);
    }
}


// ---------------------------------------------------------------------------------------
// Fused task: M operations with the same output rows whose products are added up (the channel
// sum of the graph-convolution layer, Fig. 6 / Fig. 7) in registers, so the block is written
// once instead of M times and never read back.  The set runs from its merged CSR (built once
// per plan by merge_sets_kernel below): the task is then an ordinary staged item whose dense
// tile is the members' tiles laid end to end.  Everything goes straight from global memory
// into LDS, 16 bytes per lane (the merged arrays are the library's own: aligned and padded).
// ---------------------------------------------------------------------------------------
// `vecs` 16-byte vectors global -> LDS by the whole workgroup, 1 KiB per wavefront instruction.
__device__ __forceinline__ void wg_copy_vec4(const int32_t* src, int* dst_lds, int vecs, int wave,
                                             int wl)
{
    for (int e0 = wave << 6; e0 < vecs; e0 += kThreads) {
        const int e = e0 + wl;
        if (e < vecs)
            __builtin_amdgcn_global_load_lds(
                (const void __attribute__((address_space(1)))*)(src + 4 * e),
                (void __attribute__((address_space(3)))*)(dst_lds + 4 * e0), 16, 0, 0);
    }
}

template <int VEC>
__device__ __forceinline__ void run_fused(const LaunchParams& P, int* sm, int first_item,
                                          int task)
{
    using V = Vec<VEC>;
    using VT = typename V::type;
    const int tid = threadIdx.x;
    // ---- member descriptors: lane j of every wavefront fetches member j's item, so all of
    // them arrive in one round trip; the uniform code below picks a member's fields out of
    // the lanes with v_readlane (no scalar load and no LDS per member).  The task's own
    // fields are member 0's; its rpt_off, nz_off and nnz describe the merged CSR of the set.
    const int wl = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const WorkItem mine = P.items[first_item + min(wl, P.fused_stride - 1)];
    auto lane_i32 = [](int v, int j) { return __builtin_amdgcn_readlane(v, j); };
    auto lane_i64 = [](int64_t v, int j) {
        const unsigned lo = __builtin_amdgcn_readlane((int)(v & 0xffffffff), j);
        const unsigned hi = __builtin_amdgcn_readlane((int)(v >> 32), j);
        return (int64_t)(((uint64_t)hi << 32) | lo);
    };
    const int nrows = lane_i32(mine.nrows, 0);
    if (nrows <= 0) return;
    const int staged0 = lane_i32(mine.staged, 0);
    const int m = lane_i32(mine.m, 0);
    const int fw = lane_i32(mine.fw, 0);
    const int f0 = lane_i32(mine.f0, 0);
    const int row0 = lane_i32(mine.row0, 0);
    const int nnz_sum = lane_i32(mine.nnz, 0);
    const int64_t out_row_off = lane_i64(mine.out_row_off, 0);
    const int members = (staged0 >> 8) & 0xff;
    const FusedLayout L = fused_layout(m, nnz_sum);
    const int stride = round_up(fw, 4);
    const Split<kThreads, VEC> sp(fw, tid);
    const bool direct = VEC == 4 && (sp.nvec & (sp.nvec - 1)) == 0;

    // ---- stage the merged CSR
    wg_copy_vec4(merged_words(P) + lane_i64(mine.rpt_off, 0), sm, L.rs >> 2, wave, wl);
    wg_copy_vec4(merged_words(P) + lane_i64(mine.nz_off, 0), sm + L.rs, L.entry_words >> 2, wave, wl);
    // ---- and the dense tile of every member that does not share an earlier member's
    int tile_off = L.tile_off;
    for (int j = 0; j < members; ++j) {
        const int owner = (lane_i32(mine.staged, j) >> 16) & 0xff;
        if (owner != j) continue;
        const int k = lane_i32(mine.k, j);
        float* bs = reinterpret_cast<float*>(sm + tile_off);
        const float* __restrict__ src = P.in + lane_i64(mine.in_row_off, j) * P.ld_in + f0;
        if (direct) {
            const int sh = ilog2(sp.nvec);
            const int total = k << sh;
            for (int e0 = wave << 6; e0 < total; e0 += kThreads) {
                const int e = e0 + wl;
                if (e < total)
                    __builtin_amdgcn_global_load_lds(
                        (const void __attribute__((address_space(1)))*)(
                            src + (int64_t)(e >> sh) * P.ld_in + ((e & (sp.nvec - 1)) << 2)),
                        (void __attribute__((address_space(3)))*)(bs + (e0 << 2)), 16, 0, 0);
            }
        } else {
            for (int v = sp.l; v < sp.nvec; v += sp.g_lanes)
                for (int row = sp.g; row < k; row += sp.groups)
                    store_vec<VEC>(bs + row * stride + v * VEC,
                                   load_vec<VEC>(src + (int64_t)row * P.ld_in + v * VEC));
        }
        tile_off += k * stride;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // direct-to-LDS loads landed
    __syncthreads();

    // ---- rows of the sum: the plain gather loop over the merged CSR, one store per row
    const int* crpt = sm;
    const int2* cv = reinterpret_cast<const int2*>(sm + L.rs);
    const int row_end = row0 + nrows;
    float* __restrict__ dst = P.out + out_row_off * P.ld_out + f0;
    const float* tiles = reinterpret_cast<const float*>(sm + L.tile_off);
    for (int r = row0 + sp.g; r < row_end; r += sp.groups) {
        const int p1 = min(max(crpt[r + 1], 0), nnz_sum);     // malformed pointers stay bounded
        const int p0 = min(max(crpt[r], 0), p1);
        for (int v = sp.l; v < sp.nvec; v += sp.g_lanes) {
            const float* bcol = tiles + v * VEC;
            VT acc = V::zero();
            int p = p0;
            for (; p + 3 < p1; p += 4) {
                const int2 e0 = cv[p], e1 = cv[p + 1], e2 = cv[p + 2], e3 = cv[p + 3];
                const VT b0 = load_vec<VEC>(bcol + e0.x * stride);
                const VT b1 = load_vec<VEC>(bcol + e1.x * stride);
                const VT b2 = load_vec<VEC>(bcol + e2.x * stride);
                const VT b3 = load_vec<VEC>(bcol + e3.x * stride);
                V::fma(acc, __int_as_float(e0.y), b0);
                V::fma(acc, __int_as_float(e1.y), b1);
                V::fma(acc, __int_as_float(e2.y), b2);
                V::fma(acc, __int_as_float(e3.y), b3);
            }
            for (; p < p1; ++p) {
                const int2 e = cv[p];
                V::fma(acc, __int_as_float(e.y), load_vec<VEC>(bcol + e.x * stride));
            }
            store_out<VEC>(dst + (int64_t)r * P.ld_out + v * VEC, acc);
        }
    }
}

// Merged CSR of one set of summed operations (one workgroup per set, once per plan and
// direction): row r of the set = row r of member 0, then of member 1, ... (of the members that
// have such a row: the members of a group of graphs each cover their graph's rows only); an
// entry becomes (row of the concatenated dense tiles, value).  Row pointers are clamped to the member's entry
// count and columns outside a member's tile point at its row 0, so malformed input cannot make
// the product leave its LDS.
__global__ void __launch_bounds__(kThreads)
merge_sets_kernel(const SetRecord* __restrict__ sets, const int32_t* __restrict__ rpt,
                  const int32_t* __restrict__ colids, const float* __restrict__ values,
                  int32_t* __restrict__ merged)
{
    __shared__ int partial[kThreads];
    const SetRecord& g = sets[blockIdx.x];
    const int tid = threadIdx.x;
    const int m = g.m, members = g.members;
    const int per = (m + kThreads - 1) / kThreads;
    const int r0 = min(m, tid * per), r1 = min(m, r0 + per);
    // (member j holds the set's rows row_off[j] .. row_off[j] + rows[j]: all of them for summed
    // sets, its graph's share for a group of graphs)
    auto row_range = [&](int j, int row, int& a, int& b) {
        const int r = row - g.row_off[j];
        a = b = 0;
        if ((unsigned)r >= (unsigned)g.rows[j]) return;
        const int32_t* rp = rpt + g.rpt_off[j];
        b = min(max(rp[r + 1], 0), g.nnz[j]);
        a = min(max(rp[r], 0), b);
    };
    int sum = 0;
    for (int r = r0; r < r1; ++r)
        for (int j = 0; j < members; ++j) {
            int a, b;
            row_range(j, r, a, b);
            sum += b - a;
        }
    partial[tid] = sum;
    __syncthreads();
    for (int off = 1; off < kThreads; off <<= 1) {     // inclusive scan over the lanes' sums
        const int add = tid >= off ? partial[tid - off] : 0;
        __syncthreads();
        partial[tid] += add;
        __syncthreads();
    }
    int pos = partial[tid] - sum;
    int32_t* mr = merged + g.merged_rpt_off;
    int2* mc = reinterpret_cast<int2*>(merged + g.merged_nz_off);
    // plain sets (one dense block): an ordinary CSR, columns and values in arrays of their own
    int nnz_sum = 0;
    for (int j = 0; j < members; ++j) nnz_sum += g.nnz[j];
    int32_t* pc = merged + g.merged_nz_off;
    float* pv = reinterpret_cast<float*>(pc + round_up(nnz_sum, 4));
    for (int r = r0; r < r1; ++r) {
        mr[r] = pos;
        for (int j = 0; j < members; ++j) {
            int a, b;
            row_range(j, r, a, b);
            const int32_t* ci = colids + g.nz_off[j];
            const float* va = values + g.nz_off[j];
            for (int p = a; p < b; ++p) {
                const int c = ci[p];
                const int row = g.tile_row[j] + ((unsigned)c < (unsigned)g.k[j] ? c : 0);
                if (g.plain) {
                    pc[pos] = row;
                    pv[pos] = va[p];
                } else {
                    mc[pos] = make_int2(row, __float_as_int(va[p]));
                }
                ++pos;
            }
        }
    }
    if (tid == kThreads - 1) mr[m] = pos;

    // Rows in use (groups of the streaming launch with several channels): a row of a channel's
    // dense tile that no entry of that channel names is never read, so it need not be made.
    // Per channel the rows that are named are listed in ascending order, the columns of the
    // merged CSR are renumbered to the position in the channels' lists laid end to end, and
    // behind the values go: the channels' counts, the first tile row of each channel, and the
    // lists (kxt words per channel, kxt = rows of the group's layer input).
    const int chans = g.compact & 0xff, kxt = g.compact >> 8;
    if (chans == 0) return;
    __shared__ int rank[kCompactRows];         // 1 + position of a row in its channel's list, 0: not in use
    __shared__ int base[kMaxMembers + 1];
    const int tile_rows = chans * kxt;          // (the host compacts only sets with tile_rows <= kCompactRows)
    for (int i = tid; i < tile_rows; i += kThreads) rank[i] = 0;
    __syncthreads();
    {
        int q = partial[tid] - sum;
        for (int r = r0; r < r1; ++r)
            for (int j = 0; j < members; ++j) {
                int a, b;
                row_range(j, r, a, b);
                for (int p = a; p < b; ++p) rank[pc[q++]] = 1;
            }
    }
    __syncthreads();
    int32_t* cnt = reinterpret_cast<int32_t*>(pv + round_up(nnz_sum, 4));
    int32_t* first_row = cnt + round_up(chans, 4);
    int32_t* lists = first_row + round_up(chans, 4);
    if (tid < chans) {
        int n = 0;
        for (int j = 0; j < kxt; ++j)
            if (rank[tid * kxt + j]) {
                lists[tid * kxt + n] = j;
                rank[tid * kxt + j] = ++n;
            }
        cnt[tid] = n;
        base[tid] = n;
    }
    __syncthreads();
    if (tid == 0) {
        int at = 0;
        for (int c = 0; c < chans; ++c) {
            const int n = base[c];
            base[c] = at;
            first_row[c] = at;
            at += n;
        }
    }
    __syncthreads();
    {
        int q = partial[tid] - sum;
        for (int r = r0; r < r1; ++r)
            for (int j = 0; j < members; ++j) {
                int a, b;
                row_range(j, r, a, b);
                for (int p = a; p < b; ++p, ++q) {
                    const int row = pc[q];
                    pc[q] = base[row / kxt] + rank[row] - 1;
                }
            }
    }
}

// One task of a sub-workgroup range: 256/S slots, one staged item each.
template <int LOG2S, int VEC, bool HUBS>
__device__ __forceinline__ void run_slots(const LaunchParams& P, int* sm, int first_item)
{
    constexpr int S = 1 << LOG2S;
    const int tid = threadIdx.x;
    const int slot = tid >> LOG2S;
    const int lane = tid & (S - 1);
    int idx = first_item + slot;
    if (LOG2S == 6) idx = __builtin_amdgcn_readfirstlane(idx);   // uniform inside a wavefront
    const WorkItem it = P.items[idx];
    int* slot_sm = sm + slot * (P.lds_floats >> (8 - LOG2S));
    if (it.nrows > 0) stage_item<S, VEC, HUBS>(P, it, slot_sm, lane);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // direct-to-LDS loads landed
    __syncthreads();
    if (it.nrows > 0) compute_staged<S, VEC, HUBS>(P, it, slot_sm, lane);
}


// One launch runs the whole schedule.  By default the grid has one workgroup per task (the
// hardware dispatcher balances uneven tasks, largest first); when the plan asks for fewer
// resident workgroups, workgroup w takes tasks w, w + gridDim.x, ... and fetches the next
// item's descriptor while it processes the current one.  Tasks below wg_end[0] are one item
// for the whole workgroup (bins workgroup and generic), tasks below wg_end[1] add up several
// operations into one output block, later tasks hold 4, 8 or 16 items for 64-, 32- or 16-lane
// slots.
// SLICES = false leaves out the 32- and 16-lane slot code (per-lane item descriptors cost
// registers, hence occupancy); the host launches it for schedules without such items.
// HUBS = true adds the split-row path for hub rows (an option of the plan: it costs a
// register-limited occupancy step and LDS for the reduction, which plain batches do not need).
template <int VEC, bool SLICES, bool HUBS, bool MERGED = false>
__global__ void __launch_bounds__(kThreads) bspmm_kernel(const LaunchParams P)
{
    extern __shared__ __align__(16) int sm[];
    const int tid = threadIdx.x;
    const int stride = gridDim.x;
    int t = blockIdx.x;
    if (t < P.wg_end[0]) {
        WorkItem it = P.items[P.item_base[0] + t];   // uniform address: scalar loads
        for (;;) {
            const int tn = t + stride;
            const bool more = tn < P.wg_end[0];
            WorkItem nx = it;
            if (more) nx = P.items[P.item_base[0] + tn];
            if (it.nrows > 0) {
                if (it.staged) {
                    stage_item<kThreads, VEC, HUBS, true, MERGED>(P, it, sm, tid);
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // direct-to-LDS loads landed
                    __syncthreads();
                    compute_staged<kThreads, VEC, HUBS>(P, it, sm, tid);
                } else {
                    run_generic<VEC, HUBS>(P, it, sm, tid);
                }
            }
            t = tn;
            if (!more) break;
            __syncthreads();   // the next item overwrites the LDS this one was read from
            it = nx;
        }
    }
    for (; t < P.n_tasks; t += stride) {
        __syncthreads();
        if (t < P.wg_end[1]) {
            run_fused<VEC>(P, sm, P.item_base[1] + (t - P.wg_end[0]) * P.fused_stride, t);
        } else if (t < P.wg_end[2]) {
            run_slots<6, VEC, HUBS>(P, sm, P.item_base[2] + (t - P.wg_end[1]) * 4);
        } else if (SLICES) {
            if (t < P.wg_end[3])
                run_slots<5, VEC, HUBS>(P, sm, P.item_base[3] + (t - P.wg_end[2]) * 8);
            else
                run_slots<4, VEC, HUBS>(P, sm, P.item_base[4] + (t - P.wg_end[3]) * 16);
        }
    }
}

// ---------------------------------------------------------------------------------------
// Lean launch.  When every task of a schedule is one staged workgroup item whose dense tile is
// a power-of-two number of float4 wide (molecule-sized batches: the launch fits the chip at
// once and its time is the life of a workgroup, a chain of short latencies), the launch runs
// this kernel instead of bspmm_kernel: the same staging and the same gather (Fig. 4 per row,
// batched as in Sec. IV-C, column blocking of Fig. 5(d)), with nothing on the path that such
// an item does not need.  The dense tile is requested first (it is the part that comes from
// HBM), every lane group asks for the row pointers of its own first row directly, so the first
// pass over the rows starts from registers instead of a dependent LDS read, and the address
// arithmetic of the copies is scalar wherever the item decides it.
// Results are bit for bit those of bspmm_kernel: same order of the additions inside a row.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float4 gather_row(const int2* cv, const char* bcol, int p0, int p1)
{
    using V = Vec<4>;
    float4 acc = V::zero();
    // Four entries per trip, all their LDS reads in flight together, also on the last trip of
    // a row: an entry past the end reads the row's last one and counts with value zero (the
    // sum starts at +0 and can never become -0, so adding 0 * b leaves its bits unchanged).
    const int last = p1 - 1;
    for (int p = p0; p < p1; p += 4) {
        const int2 e0 = cv[p], e1 = cv[min(p + 1, last)], e2 = cv[min(p + 2, last)],
                   e3 = cv[min(p + 3, last)];
        const float4 b0 = *reinterpret_cast<const float4*>(bcol + e0.x);
        const float4 b1 = *reinterpret_cast<const float4*>(bcol + e1.x);
        const float4 b2 = *reinterpret_cast<const float4*>(bcol + e2.x);
        const float4 b3 = *reinterpret_cast<const float4*>(bcol + e3.x);
        V::fma(acc, __int_as_float(e0.y), b0);
        V::fma(acc, p + 1 < p1 ? __int_as_float(e1.y) : 0.f, b1);
        V::fma(acc, p + 2 < p1 ? __int_as_float(e2.y) : 0.f, b2);
        V::fma(acc, p + 3 < p1 ? __int_as_float(e3.y) : 0.f, b3);
    }
    return acc;
}

// The same sum with the dense rows gathered from global memory (L2): `cv` holds (byte offset
// of the dense row inside the operation's block, value), `src_l` addresses this lane's float4 of
// the block's first row.  Four independent gathers are in flight per lane (eight measured the
// same: the gathers of a large operation are bound by what the L2 delivers, not by latency).
__device__ __forceinline__ float4 gather_row_global(const int2* cv, const char* __restrict__ src_l,
                                                    int p0, int p1)
{
    using V = Vec<4>;
    float4 acc = V::zero();
    const int last = p1 - 1;
    for (int p = p0; p < p1; p += 4) {
        int2 e[4];
        float4 b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) e[u] = cv[min(p + u, last)];
#pragma unroll
        for (int u = 0; u < 4; ++u) b[u] = *reinterpret_cast<const float4*>(src_l + (uint32_t)e[u].x);
#pragma unroll
        for (int u = 0; u < 4; ++u) V::fma(acc, p + u < p1 ? __int_as_float(e[u].y) : 0.f, b[u]);
    }
    return acc;
}

// Row block of the generic bin in a lean launch.  ONE round trip to memory brings the block's
// row pointers and its entries: their position comes with the item (lean_hints_kernel wrote it
// there once), where bspmm_kernel needs the row pointers before it can ask for the entries.
// (Fetching the block's share of the dense rows into L2 ahead of the gathers was measured and
// changed nothing: the gathers are bound by L2 throughput.)
__device__ __forceinline__ void lean_row_block(const LeanItem& it, int* sm,
                                               const int32_t* __restrict__ rpt,
                                               const int32_t* __restrict__ colids,
                                               const float* __restrict__ values,
                                               const float* __restrict__ in, float* __restrict__ out,
                                               uint32_t ld_in, uint32_t ld_out, uint32_t lds_words)
{
    const uint32_t tid = threadIdx.x;
    const int nrows = it.nrows, k = it.k, nnz = it.nnz;
    const int sh = it.sh;
    const uint32_t nvec = 1u << sh;
    const uint32_t l = tid & (nvec - 1), g = tid >> sh, groups = kThreads >> sh;
    const int pbeg = min(max(it.tile_vecs, 0), nnz);
    const int cnt = min(max(it.count, 0), nnz - pbeg);
    const uint32_t row_bytes = ld_in << 2;
    const char* __restrict__ src =
        reinterpret_cast<const char*>(in + ((uint64_t)it.in_row * ld_in + (uint32_t)it.f0));
    const int32_t* __restrict__ rp = rpt + it.rpt_off + (uint32_t)it.row0;
    const int32_t* __restrict__ ci = colids + it.nz_off + (uint32_t)pbeg;
    const float* __restrict__ va = values + it.nz_off + (uint32_t)pbeg;
    const uint32_t cv_off = (uint32_t)round_up(nrows + 1, 2);
    const bool fits = cv_off + 2u * (uint32_t)cnt <= lds_words;   // entries of the block in LDS
    int2* cv = reinterpret_cast<int2*>(sm + cv_off);

    // ---- requests
    const uint32_t ri = min(tid, (uint32_t)nrows);
    const int rv = rp[ri];
    const uint32_t last = (uint32_t)max(cnt - 1, 0);
    const uint32_t i0 = min(tid, last), i1 = min(tid + kThreads, last);
    int c0 = 0, c1 = 0;
    float a0 = 0.f, a1 = 0.f;
    if (fits && cnt > 0) {
        c0 = ci[i0];
        a0 = va[i0];
    }
    if (fits && cnt > kThreads) {
        c1 = ci[i1];
        a1 = va[i1];
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- LDS writes (clamped as in the staged path)
    sm[ri] = min(max(rv, 0), nnz);
    if (fits && cnt > 0)
        cv[i0] = make_int2((unsigned)c0 < (unsigned)k ? (int)__umul24((uint32_t)c0, row_bytes) : 0, __float_as_int(a0));
    if (fits && cnt > kThreads)
        cv[i1] = make_int2((unsigned)c1 < (unsigned)k ? (int)__umul24((uint32_t)c1, row_bytes) : 0, __float_as_int(a1));
    if (fits && cnt > 2 * kThreads)
        for (int p = tid + 2 * kThreads; p < cnt; p += kThreads) {
            const int c = ci[p];
            cv[p] = make_int2((unsigned)c < (unsigned)k ? (int)__umul24((uint32_t)c, row_bytes) : 0,
                              __float_as_int(va[p]));
        }
    __syncthreads();

    // ---- rows
    const char* src_l = src + (l << 4);
    char* __restrict__ dst = reinterpret_cast<char*>(
        out + (((uint64_t)it.out_row + (uint32_t)it.row0) * ld_out + (uint32_t)it.f0));
    const uint32_t out_row_bytes = ld_out << 2;
    for (uint32_t i = g; i < (uint32_t)nrows; i += groups) {
        const int p1 = min(max(sm[i + 1] - pbeg, 0), cnt);
        const int p0 = min(max(sm[i] - pbeg, 0), p1);
        float4 acc;
        if (fits) {
            acc = gather_row_global(cv, src_l, p0, p1);
        } else {
            // a block whose entries do not fit LDS (rows of thousands of entries): entry by
            // entry from global memory, four gathers in flight
            acc = Vec<4>::zero();
            for (int p = p0; p < p1; p += 4) {
                int cc[4];
                float aa[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int q = min(p + u, p1 - 1);
                    const int c = ci[q];
                    cc[u] = (unsigned)c < (unsigned)k ? c : 0;
                    aa[u] = p + u < p1 ? va[q] : 0.f;
                }
                float4 b[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    b[u] = *reinterpret_cast<const float4*>(src_l + __umul24((uint32_t)cc[u], row_bytes));
#pragma unroll
                for (int u = 0; u < 4; ++u) Vec<4>::fma(acc, aa[u], b[u]);
            }
        }
        store_out<4>(reinterpret_cast<float*>(dst + (__umul24(i, out_row_bytes) + (l << 4))), acc);
    }
}

// Once per plan and direction: the position of every row block's entries goes into its item.
__global__ void lean_hints_kernel(LeanItem* items, int n, const int32_t* __restrict__ rpt)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    LeanItem& it = items[i];
    if ((it.flags & 2) == 0 || it.nrows <= 0) return;
    const int32_t* rp = rpt + it.rpt_off;
    const int a = min(max(rp[it.row0], 0), it.nnz);
    const int b = min(max(rp[it.row0 + it.nrows], 0), it.nnz);
    it.tile_vecs = a;
    it.count = max(b - a, 0);
}

__global__ void __launch_bounds__(kThreads)
bspmm_lean_kernel(const LeanItem* __restrict__ items, const int32_t* __restrict__ rpt,
                  const int32_t* __restrict__ colids, const float* __restrict__ values,
                  const float* __restrict__ in, float* __restrict__ out, uint32_t ld_in,
                  uint32_t ld_out, uint32_t lds_words)
{
    extern __shared__ __align__(16) int sm[];
    const uint32_t tid = threadIdx.x;
    // One clause of scalar loads fetches the whole item; there is no early exit for an empty
    // item (all its sizes are zero, so nothing below has a trip): a branch on one field would
    // split the fetch into two dependent round trips.  The output arguments are pulled in here
    // as well, not after the barrier where they are first used.
    const LeanItem it = items[blockIdx.x];
    asm volatile("" ::"s"(out), "s"(ld_out));
    if (it.flags & 2) {        // (the same for the whole workgroup)
        lean_row_block(it, sm, rpt, colids, values, in, out, ld_in, ld_out, lds_words);
        return;
    }
    const int m = it.m, k = it.k, nnz = it.nnz;
    const int sh = it.sh;
    const uint32_t nvec = 1u << sh;                  // float4 per tile row, <= 64
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6), wl = tid & 63;
    char* lds = reinterpret_cast<char*>(sm);

    // ---- dense tile, straight from global memory into LDS, 1 KiB per wavefront instruction
    // (lane i lands at base + 16*i); a tile no other item reads is streamed.  Offsets inside
    // the item's block are 32-bit (the host launches this kernel only when they fit).
    {
        const char* __restrict__ src =
            reinterpret_cast<const char*>(in + ((uint64_t)it.in_row * ld_in + (uint32_t)it.f0));
        const uint32_t row_bytes = ld_in << 2;
        const uint32_t total = (uint32_t)it.tile_vecs;
        char* bs = lds + it.b_byte;
        if (it.flags & 1) {
            for (uint32_t e0 = wave << 6; e0 < total; e0 += kThreads) {
                const uint32_t e = e0 + wl;
                if (e < total)
                    __builtin_amdgcn_global_load_lds(
                        (const void __attribute__((address_space(1)))*)(
                            src + (__umul24(e >> sh, row_bytes) + ((e & (nvec - 1)) << 4))),
                        (void __attribute__((address_space(3)))*)(bs + (e0 << 4)), 16, 0, 2);
            }
        } else {
            for (uint32_t e0 = wave << 6; e0 < total; e0 += kThreads) {
                const uint32_t e = e0 + wl;
                if (e < total)
                    __builtin_amdgcn_global_load_lds(
                        (const void __attribute__((address_space(1)))*)(
                            src + (__umul24(e >> sh, row_bytes) + ((e & (nvec - 1)) << 4))),
                        (void __attribute__((address_space(3)))*)(bs + (e0 << 4)), 16, 0, 0);
            }
        }
    }
    // ---- CSR: the row pointers of this lane group's first row (they stay in registers), all
    // row pointers and the entries (on their way to LDS).  Indices are clamped instead of
    // predicated: a lane past the end reads, and later writes, what the last lane does.
    const int32_t* __restrict__ rp = rpt + it.rpt_off;
    const int32_t* __restrict__ ci = colids + it.nz_off;
    const float* __restrict__ va = values + it.nz_off;
    const uint32_t r_first = (uint32_t)it.row0 + (tid >> sh);
    const uint32_t um = (uint32_t)m;
    const int q0 = rp[min(r_first, um)];
    const int q1 = rp[min(r_first + 1, um)];
    const uint32_t ri = min(tid, um);
    const int rv = rp[ri];
    const uint32_t last = (uint32_t)max(nnz - 1, 0);
    const uint32_t i0 = min(tid, last), i1 = min(tid + kThreads, last);
    int c0 = 0, c1 = 0;
    float a0 = 0.f, a1 = 0.f;
    if (nnz > 0) {               // (the same for every lane: a scalar branch)
        c0 = ci[i0];
        a0 = va[i0];
    }
    if (nnz > kThreads) {
        c1 = ci[i1];
        a1 = va[i1];
    }
    // No use of a loaded value above this line (its wait would hold back later loads).
    __builtin_amdgcn_sched_barrier(0);

    // ---- LDS writes.  Row pointers are clamped to [0, nnz] and columns to [0, k): malformed
    // arrays cannot make a lane leave the item's LDS.  An entry carries the byte offset of its
    // dense row inside the tile.
    const int lsh = sh + 4;                          // log2 of the tile's row stride in bytes
    int2* cv = reinterpret_cast<int2*>(lds + it.cv_byte);
    sm[ri] = min(max(rv, 0), nnz);
    if (nnz > 0) cv[i0] = make_int2((unsigned)c0 < (unsigned)k ? c0 << lsh : 0, __float_as_int(a0));
    if (nnz > kThreads) cv[i1] = make_int2((unsigned)c1 < (unsigned)k ? c1 << lsh : 0, __float_as_int(a1));
    if (m >= kThreads)
        for (int i = tid + kThreads; i <= m; i += kThreads) sm[i] = min(max(rp[i], 0), nnz);
    if (nnz > 2 * kThreads)
        for (int p = tid + 2 * kThreads; p < nnz; p += kThreads) {
            const int c = ci[p];
            cv[p] = make_int2((unsigned)c < (unsigned)k ? c << lsh : 0, __float_as_int(va[p]));
        }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // direct-to-LDS loads landed
    __syncthreads();

    // ---- rows: the first pass from the registers, later passes from the staged row pointers
    const uint32_t l = tid & (nvec - 1);
    const char* bcol = lds + it.b_byte + (l << 4);
    char* __restrict__ dst = reinterpret_cast<char*>(out + ((uint64_t)it.out_row * ld_out + (uint32_t)it.f0));
    const uint32_t out_row_bytes = ld_out << 2;
    const uint32_t row_end = (uint32_t)(it.row0 + it.nrows);
    const uint32_t groups = kThreads >> sh;          // rows in flight
    if (r_first < row_end)
        store_out<4>(reinterpret_cast<float*>(dst + (__umul24(r_first, out_row_bytes) + (l << 4))),
                     gather_row(cv, bcol, min(max(q0, 0), nnz), min(max(q1, 0), nnz)));
    for (uint32_t r = r_first + groups; r < row_end; r += groups)
        store_out<4>(reinterpret_cast<float*>(dst + (__umul24(r, out_row_bytes) + (l << 4))),
                     gather_row(cv, bcol, sm[r], sm[r + 1]));
}

// ---------------------------------------------------------------------------------------
// transposed CSR build: one workgroup per operation.
//   count entries per column -> exclusive prefix sum (row pointers of A^T) -> scatter the
//   entry positions with atomic cursors (arrival order is arbitrary) -> every entry finds its
//   rank inside its column segment by counting the positions smaller than its own.
// The result does not depend on the arrival order: it is the stable transpose.
// `work` is k+1 counters followed by nnz positions (and, for small operations, the input's
// row pointers), in LDS when it fits, else in global scratch (both reached through flat
// addressing).
// ---------------------------------------------------------------------------------------
// FROM_COO = true sorts a SparseTensor / COO operation (index pairs as in Fig. 2:
// ids[2p] = row, ids[2p+1] = column, in any order) into CSR with the same machinery: the key is
// the row, the payload the column; `colids` is then the pair array, o.k the number of rows,
// o.m the number of columns, and the result is the stable sort by row (entries of a row keep
// their stored order).
template <bool FROM_COO, int T>
__global__ void __launch_bounds__(T)
build_sorted_kernel(const OpRecord* __restrict__ ops, const int32_t* __restrict__ rpt,
                    const int32_t* __restrict__ colids, const float* __restrict__ values,
                    int32_t* __restrict__ rpt_t, int32_t* __restrict__ colids_t,
                    float* __restrict__ values_t, int32_t* gscratch,
                    const int32_t* __restrict__ order)
{
    extern __shared__ __align__(16) int sm[];
    __shared__ int partial[T];
    // (operations are taken largest first: the launch lasts as long as its slowest workgroup)
    const OpRecord o = ops[order[blockIdx.x]];
    const int tid = threadIdx.x;
    const int k = o.k, m = o.m, nnz = o.nnz;
    int* cnt = o.scratch_off >= 0 ? gscratch + o.scratch_off : sm;   // k+1 ints
    int* pos = cnt + (k + 1);                                          // nnz ints
    const int32_t* ci = colids + (FROM_COO ? 2 * o.nz_off : o.nz_off);
    const int32_t* rp = rpt + o.rpt_off;
    int32_t* rt = rpt_t + o.rpt_t_off;
    // key of entry p, or -1 when the entry is malformed and must be skipped
    auto key_of = [&](int p) {
        if (FROM_COO) {
            const int r = ci[2 * p], c = ci[2 * p + 1];
            return ((unsigned)r < (unsigned)k && (unsigned)c < (unsigned)m) ? r : -1;
        }
        const int c = ci[p];
        return (unsigned)c < (unsigned)k ? c : -1;
    };

    // ---- small operations (flagged by the host: everything in LDS, at most four entries per
    // lane): one round trip to memory reads the operation into registers (and the row
    // pointers into LDS, which turns the search for an entry's row into LDS reads), the scan
    // runs on wavefront shuffles, and nothing is read twice.
    if (o.small == 1) {
        constexpr int E = build_entries_per_lane(T);
        int key[E], pay[E];
        float val[E];
        const float* va = values + o.nz_off;
        int* rps = pos + nnz;                              // CSR input only: m+1 row pointers
#pragma unroll
        for (int u = 0; u < E; ++u) {
            const int p = tid + u * T;
            key[u] = -1;
            pay[u] = 0;
            val[u] = 0.f;
            if (p < nnz) {
                if (FROM_COO) {
                    const int r = ci[2 * p], c = ci[2 * p + 1];
                    key[u] = ((unsigned)r < (unsigned)k && (unsigned)c < (unsigned)m) ? r : -1;
                    pay[u] = c;
                } else {
                    const int c = ci[p];
                    key[u] = (unsigned)c < (unsigned)k ? c : -1;
                }
                val[u] = va[p];
            }
        }
        if (!FROM_COO)
            for (int i = tid; i <= m; i += T) rps[i] = rp[i];
        for (int c = tid; c <= k; c += T) cnt[c] = 0;
        __syncthreads();
#pragma unroll
        for (int u = 0; u < E; ++u)
            if (key[u] >= 0) atomicAdd(&cnt[key[u] + 1], 1);
        __syncthreads();

        // inclusive scan of cnt[0..k]: a lane sums its chunk, the wavefront scans the sums with
        // shuffles, the four wavefront totals go through LDS
        const int chunk = (k + 1 + T - 1) / T;
        const int lo = tid * chunk;
        const int hi = min(lo + chunk, k + 1);
        int sum = 0;
        for (int c = lo; c < hi; ++c) sum += cnt[c];
        int incl = sum;
        const int wl = tid & 63;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int n = __shfl_up(incl, d);
            if (wl >= d) incl += n;
        }
        if (wl == 63) partial[tid >> 6] = incl;
        __syncthreads();
        int run = incl - sum;
        for (int w = 0; w < (tid >> 6); ++w) run += partial[w];
        for (int c = lo; c < hi; ++c) {
            run += cnt[c];
            cnt[c] = run;
            rt[c] = run;
        }
        __syncthreads();

        // scatter positions; cnt[c] ends as the first position of column c+1
#pragma unroll
        for (int u = 0; u < E; ++u)
            if (key[u] >= 0) pos[atomicAdd(&cnt[key[u]], 1)] = tid + u * T;
        __syncthreads();

#pragma unroll
        for (int u = 0; u < E; ++u) {
            if (key[u] < 0) continue;
            const int p = tid + u * T;
            const int c = key[u];
            const int beg = c > 0 ? cnt[c - 1] : 0;
            const int end = cnt[c];
            int rank = 0;
            for (int t = beg; t < end; ++t) rank += pos[t] < p ? 1 : 0;
            int a = pay[u];
            if (!FROM_COO) {
                // row of entry p: the last r with rp[r] <= p
                a = 0;
                int b = m;
                while (b - a > 1) {
                    const int mid = (a + b) >> 1;
                    if (rps[mid] <= p) a = mid; else b = mid;
                }
            }
            colids_t[o.nz_t_off + beg + rank] = a;
            values_t[o.nz_t_off + beg + rank] = val[u];
        }
        return;
    }

    // ---- operations of more than a thousand entries that still fit LDS (flagged 2 by the
    // host): every entry is read from memory ONCE, in order, with all loads of a lane in flight
    // together; its key and its payload - for CSR input the row, which a pass over the row
    // pointers ORs in - are packed into one LDS word, so the histogram, the scatter and the
    // ranking run out of LDS, and the last pass walks the entries in stored order again
    // (coalesced value loads; the scattered side is the stores, which nothing waits for).
    if (o.small == 2) {
        const int kb = 32 - __clz(k);                     // bits of a key; the value k marks a skipped entry
        const unsigned kmask = (1u << kb) - 1u;
        unsigned* keyrow = reinterpret_cast<unsigned*>(pos + nnz);
        for (int c = tid; c <= k; c += T) cnt[c] = 0;
        __syncthreads();
        for (int p0 = tid; p0 < nnz; p0 += 4 * T) {
            int key[4], pay[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int p = p0 + u * T;
                key[u] = k;
                pay[u] = 0;
                if (p < nnz) {
                    if (FROM_COO) {
                        const int r = ci[2 * p], c = ci[2 * p + 1];
                        if ((unsigned)r < (unsigned)k && (unsigned)c < (unsigned)m) key[u] = r;
                        pay[u] = c;
                    } else {
                        const int c = ci[p];
                        if ((unsigned)c < (unsigned)k) key[u] = c;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int p = p0 + u * T;
                if (p < nnz) {
                    keyrow[p] = (unsigned)key[u] | (key[u] < k ? (unsigned)pay[u] << kb : 0u);
                    if (key[u] < k) atomicAdd(&cnt[key[u] + 1], 1);
                }
            }
        }
        if (!FROM_COO) {
            __syncthreads();          // keys in place before the rows are ORed in
            for (int r = tid; r < m; r += T) {
                const int b = min(max(rp[r + 1], 0), nnz);
                const int a = min(max(rp[r], 0), b);
                for (int p = a; p < b; ++p) atomicOr(&keyrow[p], (unsigned)r << kb);
            }
        }
        __syncthreads();

        // inclusive scan of cnt[0..k] (as below)
        const int chunk = (k + 1 + T - 1) / T;
        const int lo = tid * chunk;
        const int hi = min(lo + chunk, k + 1);
        int sum = 0;
        for (int c = lo; c < hi; ++c) sum += cnt[c];
        int incl = sum;
        const int wl = tid & 63;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int n = __shfl_up(incl, d);
            if (wl >= d) incl += n;
        }
        if (wl == 63) partial[tid >> 6] = incl;
        __syncthreads();
        int run = incl - sum;
        for (int w = 0; w < (tid >> 6); ++w) run += partial[w];
        for (int c = lo; c < hi; ++c) {
            run += cnt[c];
            cnt[c] = run;
            rt[c] = run;
        }
        __syncthreads();

        // scatter positions; cnt[c] ends as the first position of key c+1
        for (int p = tid; p < nnz; p += T) {
            const int c = (int)(keyrow[p] & kmask);
            if (c < k) pos[atomicAdd(&cnt[c], 1)] = p;
        }
        __syncthreads();

        const float* va = values + o.nz_off;
        float v_next = tid < nnz ? va[tid] : 0.f;
        for (int p = tid; p < nnz; p += T) {
            const float v = v_next;
            if (p + T < nnz) v_next = va[p + T];     // in flight during this trip
            const unsigned kr = keyrow[p];
            const int c = (int)(kr & kmask);
            if (c >= k) continue;
            const int beg = c > 0 ? cnt[c - 1] : 0;
            const int end = cnt[c];
            int rank = 0;
            for (int t = beg; t < end; ++t) rank += pos[t] < p ? 1 : 0;
            colids_t[o.nz_t_off + beg + rank] = (int)(kr >> kb);
            values_t[o.nz_t_off + beg + rank] = v;
        }
        return;
    }

    for (int c = tid; c <= k; c += T) cnt[c] = 0;
    __syncthreads();
    for (int p = tid; p < nnz; p += T) {
        const int c = key_of(p);
        if (c >= 0) atomicAdd(&cnt[c + 1], 1);
    }
    __syncthreads();

    // inclusive scan of cnt[0..k]: afterwards cnt[c] = first position of column c
    const int chunk = (k + 1 + T - 1) / T;
    const int lo = tid * chunk;
    const int hi = lo + chunk < k + 1 ? lo + chunk : k + 1;
    int sum = 0;
    for (int c = lo; c < hi; ++c) sum += cnt[c];
    partial[tid] = sum;
    __syncthreads();
    for (int d = 1; d < T; d <<= 1) {
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
    for (int p = tid; p < nnz; p += T) {
        const int c = key_of(p);
        if (c >= 0) pos[atomicAdd(&cnt[c], 1)] = p;
    }
    __syncthreads();

    const float* va = values + o.nz_off;
    const int placed = cnt[k];                      // entries that were not skipped
    for (int q = tid; q < placed; q += T) {
        const int p = pos[q];
        const int c = key_of(p);
        const int beg = c > 0 ? cnt[c - 1] : 0;
        const int end = cnt[c];
        int rank = 0;
        for (int t = beg; t < end; ++t) rank += pos[t] < p ? 1 : 0;
        int a;
        if (FROM_COO) {
            a = ci[2 * p + 1];                        // the payload is the column
        } else {
            // row of entry p: the last r with rp[r] <= p
            a = 0;
            int b = m;   // invariant: rp[a] <= p, and (b == m or rp[b] > p)
            while (b - a > 1) {
                const int mid = (a + b) >> 1;
                if (rp[mid] <= p) a = mid; else b = mid;
            }
        }
        colids_t[o.nz_t_off + beg + rank] = a;
        values_t[o.nz_t_off + beg + rank] = va[p];
    }
}

// Index pairs of a COO operation inside their matrix?
__global__ void __launch_bounds__(kThreads)
validate_coo_kernel(const OpRecord* __restrict__ ops, const int32_t* __restrict__ ids, int32_t* flag)
{
    const OpRecord o = ops[blockIdx.x];
    const int32_t* id = ids + 2 * o.nz_off;
    bool bad = false;
    for (int p = threadIdx.x; p < o.nnz; p += kThreads)
        if ((unsigned)id[2 * p] >= (unsigned)o.k || (unsigned)id[2 * p + 1] >= (unsigned)o.m) bad = true;
    if (bad) atomicMin(flag, (int)blockIdx.x);
}

// ---------------------------------------------------------------------------------------
// One channel of the batched graph-convolution layer in one launch (Fig. 7: MatMul, Add,
// BatchedSpMM): Y_i (+)= A_i (X_i W + bias).  A workgroup stages A_i, the layer input X_i
// (k x n_front), the weight tile W[:, f0:f0+fw] and the bias tile in LDS in ONE round trip to
// memory (more when X_i does not fit at once), computes the dense tile B = X_i W + bias on the matrix cores out of LDS into the
// tile's usual place, and then runs the ordinary row gather over it: U, B and the per-channel
// C never exist in memory.
// The dense part is v_mfma_f32_16x16x4_f32 (fp32 in, fp32 accumulate).  The tile is cut into
// 16 x 16 blocks dealt to the four wavefronts.  Operand layout of the instruction: lane l
// supplies A[l % 16][l / 16] and B[l / 16][l % 16] and receives rows 4*(l / 16) .. +3 of column
// l % 16.  A lane reads four consecutive k of its X row with one 16-byte LDS read and feeds
// them to four instructions together with the weights of the same four k, so the k order
// inside a step differs from memory order for both operands alike, which leaves the product
// unchanged.
// (Whole layers in launches of several rounds use v_mfma_f32_32x32x2_f32 on 32 x 32 blocks
// instead; see dense_rows32 in the kernel.)
// LDS, in words: the staged layout of the item (row pointers, entries, dense tile k x fw),
// then the weight tile (n_front x fw), the bias tile (fw) and as many rows of X_i as fit
// (a multiple of 16; operations with more rows take several passes).
// Needs F % 16 == 0, n_front % 4 == 0 and 16-byte aligned operands (checked on the host).
// ---------------------------------------------------------------------------------------

// rows x (4 * nvec) floats, global (leading dimension ld) -> LDS (rows packed).  Whole
// wavefronts copy 1 KiB per instruction straight into LDS when a row is a power-of-two number
// of float4; otherwise through registers, four rows per lane group in flight.
// `swz` != 0 (only with a power-of-two nvec, swz < nvec) stores the float4 with index v of row r
// in slot v ^ (r & swz): rows that are a multiple of 64 words apart then no longer fall on the
// same LDS banks when 16 lanes read the same column of 16 consecutive rows.
template <int THREADS = kThreads>
__device__ __forceinline__ void stage_tile4(float* dst, const float* __restrict__ src, int64_t ld,
                                            int rows, int nvec, int tid, int swz = 0)
{
    if ((nvec & (nvec - 1)) == 0) {
        const int sh = ilog2(nvec);
        const int total = rows << sh;
        const int wl = tid & 63;
        for (int e0 = (tid >> 6) << 6; e0 < total; e0 += THREADS) {
            const int e = e0 + wl;
            if (e < total) {
                const int r = e >> sh;
                const float* gp = src + (int64_t)r * ld + ((((e & (nvec - 1)) ^ (r & swz))) << 2);
                __builtin_amdgcn_global_load_lds(
                    (const void __attribute__((address_space(1)))*)gp,
                    (void __attribute__((address_space(3)))*)(dst + (e0 << 2)), 16, 0, 0);
            }
        }
    } else {
        const int gl = min(64, pow2_ceil(nvec));
        const int sh = ilog2(gl);
        const int g = tid >> sh, l = tid & (gl - 1), G = THREADS >> sh;
        if (l < nvec)
            for (int r0 = g; r0 < rows; r0 += 4 * G) {
                float4 t[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    t[u] = load_vec<4>(src + (int64_t)min(r0 + u * G, rows - 1) * ld + 4 * l);
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (r0 + u * G < rows) store_vec<4>(dst + (r0 + u * G) * (nvec << 2) + 4 * l, t[u]);
            }
    }
}

// SETS = true: every item stands in for a set of M channel operations that share the layer
// input X_i and are summed into one output block (the whole layer of Fig. 7 in one launch):
// the dense tile is [X_i W[0] + bias[0]; ...; X_i W[M-1] + bias[M-1]] (M x kx rows), the CSR is
// the set's merged one, whose entries of channel c name rows c*kx ... of that tile; W is the M
// weight matrices one under the other (M*nx rows), bias M rows of P.fused_stride floats apart, and
// P.rpt is the base of the merged arrays.
// THREADS: 256, or 512 for launches of a single round of workgroups, whose time is the time of
// the largest item: twice the wavefronts halve its matrix blocks per wavefront and the passes
// of its gather.
template <bool ACC, bool SETS, int THREADS = kThreads>
__global__ void __launch_bounds__(THREADS) bspmm_gcn_kernel(const LaunchParams P)
{
    extern __shared__ __align__(16) int sm[];
    typedef float mfma4 __attribute__((ext_vector_type(4)));
    const int tid = threadIdx.x;
    const WorkItem it = P.items[blockIdx.x];
    if (it.nrows <= 0) return;
    const int nx = P.n_front;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), wl = tid & 63;
    const int col = wl & 15, g = wl >> 4;
    const int nb_count = it.fw >> 4;
    const int M = SETS ? max(1, (it.staged >> 8) & 0xff) : 1;   // channels
    const int kx = SETS ? it.k / M : it.k;                       // rows of X_i

    const StagedLayout L = staged_layout(it.m, it.k, it.nnz, it.fw, 0, false);
    float* bt = reinterpret_cast<float*>(sm + L.b_off);      // dense tile k x fw, made below
    float* ws = bt + it.k * it.fw;                            // weight tiles, M x (nx x fw)
    float* bias_s = ws + M * nx * it.fw;                      // bias tiles, M x fw
    float* xs = bias_s + M * it.fw;                           // rows of X_i, R x nx
    // X_i is taken R rows at a time: all of them when the rest of the LDS holds them, else a
    // multiple of 16 (a 16 x 16 block needs 16 rows of X_i and all of their columns).  The
    // host has made sure of 16.
    const int x_room = (P.lds_floats - (int)(xs - reinterpret_cast<float*>(sm))) / nx;
    const int R = kx <= x_room ? kx : x_room & ~15;
    const int xvec = nx >> 2;
    const int swz = (xvec & (xvec - 1)) == 0 ? min(xvec, 16) - 1 : 0;
    const float* xg = P.in + it.in_row_off * P.ld_in;

    // dense tile rows r0 .. r0+rows on the matrix cores, LDS -> LDS
    auto dense_rows = [&](int r0, int rows) {
        const int per_channel = ((rows + 15) >> 4) * nb_count;
        const int blocks = per_channel * M;
        for (int blk = wave; blk < blocks; blk += THREADS / 64) {
            const int c = SETS ? blk / per_channel : 0;
            const int rem = blk - c * per_channel;
            const int mb = rem / nb_count, nb = rem - mb * nb_count;
            const float bv = bias_s[c * it.fw + 16 * nb + col];
            // four independent accumulators (one per k of a lane's four): a chain of
            // dependent matrix instructions would run at their latency, not their rate
            mfma4 acc = {bv, bv, bv, bv};
            mfma4 acc1 = {0.f, 0.f, 0.f, 0.f}, acc2 = acc1, acc3 = acc1;
            const int arow = min(16 * mb + col, rows - 1);     // rows past the end repeat the last
            const float* xrow = xs + arow * nx;
            const int xs_swz = arow & swz;
            const float* wcol = ws + (c * nx + 4 * g) * it.fw + 16 * nb + col;
            // Sixteen k per trip (four per lane group, one matrix instruction each).  The
            // operands of the next trip are read from LDS before the instructions of this one
            // are issued: read latency then hides behind the matrix pipeline instead of
            // adding to every trip.
            const int nfull = nx & ~15;
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
            float w0 = 0.f, w1 = 0.f, w2 = 0.f, w3 = 0.f;
            if (nfull > 0) {
                a = *reinterpret_cast<const float4*>(xrow + ((g ^ xs_swz) << 2));
                w0 = wcol[0], w1 = wcol[it.fw], w2 = wcol[2 * it.fw], w3 = wcol[3 * it.fw];
            }
            for (int k0 = 0; k0 < nfull; k0 += 16) {
                float4 an = a;
                float v0 = w0, v1 = w1, v2 = w2, v3 = w3;
                if (k0 + 16 < nfull) {
                    an = *reinterpret_cast<const float4*>(xrow + (((((k0 + 16) >> 2) + g) ^ xs_swz) << 2));
                    const float* wk = wcol + (k0 + 16) * it.fw;
                    v0 = wk[0], v1 = wk[it.fw], v2 = wk[2 * it.fw], v3 = wk[3 * it.fw];
                }
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, w0, acc, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, w1, acc1, 0, 0, 0);
                acc2 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, w2, acc2, 0, 0, 0);
                acc3 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, w3, acc3, 0, 0, 0);
                a = an;
                w0 = v0, w1 = v1, w2 = v2, w3 = v3;
            }
            if (nfull < nx) {
                // the last, partial trip: every lane takes part in the matrix instruction; a
                // lane group whose four k lie past the end (nx % 4 == 0: all four or none)
                // reads the last valid ones instead and contributes zeros
                const bool ok = nfull + 4 * g < nx;
                const int kc = ok ? nfull : nx - 4 - 4 * g;
                float4 at = *reinterpret_cast<const float4*>(xrow + ((((kc >> 2) + g) ^ xs_swz) << 2));
                if (!ok) at = make_float4(0.f, 0.f, 0.f, 0.f);
                const float* wk = wcol + kc * it.fw;
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(at.x, wk[0], acc, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(at.y, wk[it.fw], acc1, 0, 0, 0);
                acc2 = __builtin_amdgcn_mfma_f32_16x16x4f32(at.z, wk[2 * it.fw], acc2, 0, 0, 0);
                acc3 = __builtin_amdgcn_mfma_f32_16x16x4f32(at.w, wk[3 * it.fw], acc3, 0, 0, 0);
            }
            acc = (acc + acc1) + (acc2 + acc3);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = 16 * mb + 4 * g + i;
                if (row < rows) bt[(c * kx + r0 + row) * it.fw + 16 * nb + col] = acc[i];
            }
        }
    };

    // The same on 32 x 32 blocks (channel sets whose tile is a multiple of 32 columns wide, where
    // the host asks for it with bit 3 of `staged`): a
    // block-trip of 16 k is eight matrix instructions of 64 cycles each fed by two 16-byte
    // reads of X_i and eight reads of W per lane - half the LDS reads per flop of the 16 x 16
    // form, and four times the matrix time per trip to hide their latency behind.  The
    // instruction sums over k in any order: lane half h takes k0 + 8h ... k0 + 8h + 7, which
    // are contiguous in the row of X_i.
    auto dense_rows32 = [&](int r0, int rows) {
        typedef float mfma16 __attribute__((ext_vector_type(16)));
        const int nb32 = it.fw >> 5;
        const int per_channel = ((rows + 31) >> 5) * nb32;
        const int blocks = per_channel * M;
        const int c32 = wl & 31, h = wl >> 5;
        for (int blk = wave; blk < blocks; blk += THREADS / 64) {
            const int c = blk / per_channel;
            const int rem = blk - c * per_channel;
            const int mb = rem / nb32, nb = rem - mb * nb32;
            const float bv = bias_s[c * it.fw + 32 * nb + c32];
            mfma16 acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = bv;
            const int arow = min(32 * mb + c32, rows - 1);     // rows past the end repeat the last
            const float* xrow = xs + arow * nx;
            const int xs_swz = arow & swz;
            const float* wcol = ws + (c * nx + 8 * h) * it.fw + 32 * nb + c32;
            const int nfull = nx & ~15;
            float4 a0 = make_float4(0.f, 0.f, 0.f, 0.f), a1 = a0;
            float w[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            if (nfull > 0) {
                a0 = *reinterpret_cast<const float4*>(xrow + (((2 * h) ^ xs_swz) << 2));
                a1 = *reinterpret_cast<const float4*>(xrow + (((2 * h + 1) ^ xs_swz) << 2));
#pragma unroll
                for (int j = 0; j < 8; ++j) w[j] = wcol[j * it.fw];
            }
            for (int k0 = 0; k0 < nfull; k0 += 16) {
                float4 n0 = a0, n1 = a1;
                float v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = w[j];
                if (k0 + 16 < nfull) {      // the next trip's operands, before this trip's instructions
                    const int q = ((k0 + 16) >> 2) + 2 * h;
                    n0 = *reinterpret_cast<const float4*>(xrow + ((q ^ xs_swz) << 2));
                    n1 = *reinterpret_cast<const float4*>(xrow + (((q + 1) ^ xs_swz) << 2));
                    const float* wk = wcol + (k0 + 16) * it.fw;
#pragma unroll
                    for (int j = 0; j < 8; ++j) v[j] = wk[j * it.fw];
                }
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.x, w[0], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.y, w[1], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.z, w[2], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.w, w[3], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.x, w[4], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.y, w[5], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.z, w[6], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.w, w[7], acc, 0, 0, 0);
                a0 = n0, a1 = n1;
#pragma unroll
                for (int j = 0; j < 8; ++j) w[j] = v[j];
            }
            if (nfull < nx) {
                // the last, partial trip (4, 8 or 12 k): a lane whose k lies past the end reads
                // the row's first element instead and contributes zero
                const int left = nx - nfull;
                for (int j = 0; j < min(8, left); ++j) {
                    const bool ok = 8 * h + j < left;
                    const int k = ok ? nfull + 8 * h + j : 0;
                    float av = xrow[(((k >> 2) ^ xs_swz) << 2) + (k & 3)];
                    if (!ok) av = 0.f;
                    const float wv = ws[(c * nx + k) * it.fw + 32 * nb + c32];
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av, wv, acc, 0, 0, 0);
                }
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int row = 32 * mb + 8 * (i >> 2) + 4 * h + (i & 3);
                if (row < rows) bt[(c * kx + r0 + row) * it.fw + 32 * nb + c32] = acc[i];
            }
        }
    };
    const bool blocks32 = SETS && (it.staged & 8) != 0 && (it.fw & 31) == 0;

    // ---- first pass: everything read from memory is requested at once (the first rows of
    // X_i, the weights, the bias, A_i)
    stage_tile4<THREADS>(xs, xg, P.ld_in, min(R, kx), xvec, tid, swz);
    stage_tile4<THREADS>(ws, P.w + it.f0, P.ld_w, M * nx, it.fw >> 2, tid);
    float bias_v = 0.f;
    if (tid < it.fw) bias_v = P.bias[it.f0 + tid];
    if (SETS) {
        LaunchParams Q = P;                                   // CSR from the merged arrays
        Q.w = reinterpret_cast<const float*>(P.rpt);
        stage_item<THREADS, 4, false, false, true>(Q, it, sm, tid);
        for (int e = tid + it.fw; e < M * it.fw; e += THREADS) {   // the other channels' bias
            const int c = e / it.fw;
            bias_s[e] = P.bias[(int64_t)c * P.fused_stride + it.f0 + (e - c * it.fw)];
        }
    } else {
        stage_item<THREADS, 4, false, false>(P, it, sm, tid);    // A_i only
    }
    if (tid < it.fw) bias_s[tid] = bias_v;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // direct-to-LDS loads landed
    __syncthreads();
    if (blocks32)
        dense_rows32(0, min(R, kx));
    else
        dense_rows(0, min(R, kx));
    __syncthreads();         // the rows of X_i may be replaced; after the last pass: tile complete
    // ---- operations with more rows than fit: further passes
    for (int r0 = R; r0 < kx; r0 += R) {
        const int rows = min(R, kx - r0);
        stage_tile4<THREADS>(xs, xg + (int64_t)r0 * P.ld_in, P.ld_in, rows, xvec, tid, swz);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (blocks32)
            dense_rows32(r0, rows);
        else
            dense_rows(r0, rows);
        __syncthreads();
    }
    compute_staged<THREADS, 4, false, ACC>(P, it, sm, tid);
}

// ---------------------------------------------------------------------------------------
// The layer (Fig. 7: one channel, or all channels with the ElementWiseAdd) for batches of two
// and more workgroups per CU: resident workgroups, each bound to one feature tile, stream the
// graphs of their list.  A graph is a set of M channel operations with one merged CSR block
// (row pointers, columns, values back to back); plans of single channels have such a block per
// operation (M = 1).
//
// A workgroup of bspmm_gcn_kernel goes through its phases one after the other - operands from
// memory, dense tile on the matrix cores, gather, store - stages its weight tile again for
// every graph, and the launch's LDS is sized for the largest graph of the batch.  Here
//   * the weights of a wavefront's blocks live in REGISTERS for the whole launch: wavefront w
//     owns U of the M * fw/16 (channel, 16-column block) pairs, and the B operand of
//     v_mfma_f32_16x16x4_f32 for lane (g, col) = (l / 16, l % 16) is W[ch][16 s + 4 g + j][col],
//     s < n_X / 16, j < 4: n_X / 4 registers per pair.  No LDS for W, no LDS reads for it.
//   * the rows of X_i and the merged CSR block of the NEXT graph are requested (global -> LDS
//     directly) before the matrix instructions of this graph are issued, into the other one of
//     two buffers, and nothing waits for them until the top of the next trip; a graph's results
//     wait in registers and are stored at the top of the next trip, so that wait finds only
//     requests and stores that are a whole trip old.  The records of the graphs (32 bytes
//     each) are fetched with scalar loads two trips ahead.
//   * the launch's LDS is sized for the graphs that fit a budget of a third of a CU's LDS, so
//     that three workgroups share a CU: one's matrix phase overlaps the others' gathers and
//     requests.  (Workgroups of eight wavefronts, WV = 8, which give each of eight channels a
//     wavefront of its own: half a CU's LDS, two per CU.)  Larger graphs (a few per cent of a molecule batch) are taken one at a time
//     out of the same LDS, their X_i in chunks (see below); what does not fit even so is not
//     in the lists at all (the host gives it to bspmm_gcn_kernel in a launch of its own).
// Arithmetic: the n_X products of a dense element are added by the matrix instructions in
// the order 4 g + j within 16 s (bias as the initial value of the accumulator; two
// accumulators per block, k even and odd, in kernels with one block per wavefront and in the
// halves); a row's entries are added in stored order with fused multiply-adds.  Rows of X_i
// are XOR-swizzled in LDS as in bspmm_gcn_kernel.
// Per trip two barriers: "tile free, buffers of the graph after next free, this graph's
// operands landed" and "tile complete".  Every workgroup's loop runs over a list the host
// made: it ends.
// ---------------------------------------------------------------------------------------

// Global -> LDS copy of 16 bytes per lane (lane i lands at lds + 16 i), issued from inline
// assembly: the compiler then does not know that LDS is written behind its back and does not
// put a wait for ALL outstanding memory operations in front of the next LDS read.  That wait is
// what a prefetch into the other buffer must not meet; the kernel waits for its requests
// itself, where it needs them.  (Untracked requests can only make the waits the compiler
// computes for its own loads longer, never shorter: the counter runs in issue order.)
__device__ __forceinline__ void lds_dma16(const void* gp, const void* lds)
{
    const int m0 = __builtin_amdgcn_readfirstlane(
        (int)(uintptr_t)((const __attribute__((address_space(3))) char*)lds));
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :: "v"(gp), "s"(m0) : "memory", "m0");
}

// The same with the LDS address as a number: a loop that adds to it spares the pointer
// conversion of every trip.
__device__ __forceinline__ int lds_address(const void* lds)
{
    return (int)(uintptr_t)((const __attribute__((address_space(3))) char*)lds);
}

__device__ __forceinline__ void lds_dma16_to(const void* gp, int lds_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :: "v"(gp), "s"(lds_addr) : "memory", "m0");
}

// Workgroup barrier that orders LDS accesses only (no wait for global stores or for requests
// in flight, which __syncthreads would add).
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int NX16, int U, int WV>
__global__ void __launch_bounds__(64 * WV)
bspmm_gcn_stream_kernel(const StreamSet* __restrict__ sets, const int32_t* __restrict__ list,
                        const int32_t* __restrict__ merged, const float* __restrict__ x,
                        const float* __restrict__ wgt, const float* __restrict__ bias,
                        float* __restrict__ y, const StreamShape S)
{
    extern __shared__ __align__(16) int sm[];
    typedef float mfma4 __attribute__((ext_vector_type(4)));
    constexpr int NX = 16 * NX16, XVEC = NX / 4, XSH = NX16 == 1 ? 2 : (NX16 == 2 ? 3 : (NX16 == 4 ? 4 : 5));
    constexpr int SWZ = (XVEC < 16 ? XVEC : 16) - 1;
    constexpr int T = 64 * WV;                    // lanes of the workgroup (four or eight wavefronts)
    constexpr int C = U == 1 ? 2 : 1;            // accumulators per block: two matrix instructions
                                                 // between dependent ones either way
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), wl = tid & 63;
    const int col = wl & 15, g = wl >> 4;
    // Workgroups go to the XCDs round robin (index mod 8).  The workgroups of one list - one per
    // feature tile - read the same rows of X: they sit on one XCD, so that its L2 fetches them once
    // (list = 8 * (slot / tiles) + xcd, tile = slot % tiles; the grid is padded to whole rounds).
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int tile_idx = slot % S.tiles, lp = (slot / S.tiles) * 8 + xcd;
    if (lp >= S.lists) return;
    const int f0 = tile_idx * S.fw;
    const int j0 = list[lp], j1 = list[lp + 1];
    if (j0 >= j1) return;
    const int fsh = ilog2(S.fw);                 // tile row = 1 << fsh floats
    const int nbw = S.fw >> 4;                   // 16-column blocks per tile row

    float* tile = reinterpret_cast<float*>(sm);
    float* xbase = tile + S.tile_words;
    int* cbase = sm + S.tile_words + 2 * S.x_words;
    float* sink = reinterpret_cast<float*>(cbase + 2 * S.csr_words) + wl;   // rows past the end land here

    // ---- this wavefront's weights and bias, once
    float w[U][NX16][4];
    float bv[U];
    int unit_ch[U], unit_col[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int unit = wave * U + u;
        const int ch = unit / nbw, nb = unit - ch * nbw;
        unit_ch[u] = ch;
        unit_col[u] = 16 * nb + col;
        // (a channel past the layer's own - the layer runs padded to 4 or 8 - has no weights)
        const bool live = ch < S.real_channels;
        const float* wp = wgt + (int64_t)((live ? ch : 0) * NX + 4 * g) * S.ld_w + f0 + 16 * nb + col;
#pragma unroll
        for (int s = 0; s < NX16; ++s)
#pragma unroll
            for (int j = 0; j < 4; ++j) w[u][s][j] = live ? wp[(int64_t)(16 * s + j) * S.ld_w] : 0.f;
        bv[u] = live ? bias[(int64_t)ch * S.bias_stride + f0 + 16 * nb + col] : 0.f;
    }

    // rows of X_i and the merged CSR block of a graph -> buffers b.  A lane's element of a
    // request is T elements (T / XVEC rows) after its element of the previous one: the row
    // advances by a multiple of the swizzle period, so the swizzled column is the lane's for good
    // and between requests a lane's address moves by a fixed step, like the LDS address of the
    // wavefront (the loops below are a handful of instructions a request: the wavefronts of the
    // workgroups beside this one are busy on the same SIMD, and every instruction waits its turn).
    // n_X = 128 with four wavefronts takes 8 rows a request, half a period: the swizzled column
    // flips between two places, 128 bytes apart.
    constexpr int kRowsPerRequest = T / XVEC;
    constexpr bool kFlip = kRowsPerRequest % (SWZ + 1) != 0;
    static_assert(!kFlip || (XVEC == 32 && kRowsPerRequest == 8), "swizzle period");
    const int x_row0 = tid >> XSH;
    const int x_col0 = (tid & (XVEC - 1)) ^ (x_row0 & SWZ);
    const int64_t x_lane_off = (int64_t)x_row0 * S.ld_x + (x_col0 << 2);
    const int64_t x_step = (int64_t)kRowsPerRequest * S.ld_x * 4;            // bytes
    const int x_flip = kFlip ? ((x_col0 & 8) ? -128 : 128) : 0;              // bytes, to the other place
    const int w16 = wave << 10;                                              // this wavefront's place in a request
    const int xbase_lds = lds_address(xbase) + w16, cbase_lds = lds_address(cbase) + w16;
    auto request = [&](const StreamSet& st, int b) {
        const char* gp = reinterpret_cast<const char*>(x + st.in_row * S.ld_x + x_lane_off);
        int to = xbase_lds + b * (S.x_words << 2);
        int64_t step = x_step + x_flip;
        // (left: elements of the request from this wavefront's first lane on)
        for (int left = (st.kx << XSH) - (wave << 6); left > 0; left -= T) {
            if (wl < left) lds_dma16_to(gp, to);
            gp += step;
            if (kFlip) step = 2 * x_step - step;
            to += T * 16;
        }
        const int csr_vecs = (((st.m + 4) & ~3) + 2 * ((st.nnz + 3) & ~3) +
                              (S.compact ? compact_words(S.channels, st.kx) : 0)) >> 2;
        const char* cg = reinterpret_cast<const char*>(merged + st.csr_off) + (tid << 4);
        to = cbase_lds + b * (S.csr_words << 2);
        for (int left = csr_vecs - (wave << 6); left > 0; left -= T) {
            if (wl < left) lds_dma16_to(cg, to);
            cg += T * 16;
            to += T * 16;
        }
    };

    // gather geometry: fw / 4 lanes per output row
    const int gsh = fsh - 2;
    const int r_lane = tid >> gsh, l = tid & ((1 << gsh) - 1);
    const int rows_per_pass = T >> gsh;
    float4 yv[kStreamPasses];
    int pend_m = 0;
    int64_t pend_row = 0;
    auto store_pending = [&]() {
#pragma unroll
        for (int q = 0; q < kStreamPasses; ++q) {
            const int r = q * rows_per_pass + r_lane;
            if (r < pend_m) {
                float* yp = y + (pend_row + r) * S.ld_y + f0 + 4 * l;
                float4 v = yv[q];
                if (S.accumulate) {
                    const float4 old = *reinterpret_cast<const float4*>(yp);
                    v.x += old.x, v.y += old.y, v.z += old.z, v.w += old.w;
                }
                store_out<4>(yp, v);
            }
        }
    };

    // ---- graphs too large for the buffers above come first in a list and are taken one at a
    // time, without prefetch: the tile sits at the start of LDS, the merged CSR block at its end,
    // and the rows of X_i pass through the space between them in chunks of as many 16-row blocks
    // as fit.  Kernels with two blocks per wavefront (tiles of 32 columns: a wavefront owns one
    // channel) take such a graph in two halves of 16 columns, each with a half tile
    // (channels x kx x 16); kernels with one block per wavefront take it in one piece.
    // Each piece: [chunk from memory, its blocks on the matrix cores] ..., gather, store.
    int jn = j0;
    constexpr int PIECES = U == 2 ? 2 : 1;
    if (U == 1 || nbw == 2) {
        const int psh = U == 2 ? 4 : fsh;           // a piece's tile row = 1 << psh floats
        const int total_words = S.tile_words + 2 * S.x_words + 2 * S.csr_words;
        int* cbig = sm + total_words - S.big_csr_words;
        for (; jn < j1; ++jn) {
            const StreamSet bg = sets[jn];
            const int csr_w = ((bg.m + 4) & ~3) + 2 * ((bg.nnz + 3) & ~3);
            const bool big = S.channels * bg.kx * S.fw > S.tile_words || bg.kx * NX > S.x_words ||
                             csr_w + (S.compact ? compact_words(S.channels, bg.kx) : 0) > S.csr_words ||
                             bg.m > kStreamPasses * rows_per_pass ||
                             (S.compact && S.channels * bg.kx > kCompactRows);
            if (!big) break;
            const int kx = bg.kx, m = bg.m;
            const int piece_words = (S.channels * kx) << psh;
            float* xbig = tile + piece_words;
            const int rows_chunk = min((kx + 15) & ~15, ((total_words - S.big_csr_words - piece_words) / NX) & ~15);
            if (rows_chunk < 16 || csr_w > S.big_csr_words) return;    // (the host never lists such a graph)
            {
                const int32_t* cg = merged + bg.csr_off;
                const int csr_vecs = csr_w >> 2;
                for (int e0 = wave << 6; e0 < csr_vecs; e0 += T) {
                    const int e = e0 + wl;
                    if (e < csr_vecs) lds_dma16(cg + 4 * e, cbig + (e0 << 2));
                }
            }
            const float* xg = x + bg.in_row * S.ld_x;
            const int* rp = cbig;
            const int* cols = rp + ((m + 4) & ~3);
            const float* vals = reinterpret_cast<const float*>(cols + ((bg.nnz + 3) & ~3));
#pragma unroll
            for (int h = 0; h < PIECES; ++h) {
                const int pcol = U == 2 ? col : unit_col[0];      // column inside the piece
                for (int r0 = 0; r0 < kx; r0 += rows_chunk) {
                    const int rows = min(rows_chunk, kx - r0);
                    const int total = rows << XSH;
                    for (int e0 = wave << 6; e0 < total; e0 += T) {
                        const int e = e0 + wl;
                        if (e < total) {
                            const int r = e >> XSH;
                            lds_dma16(xg + (int64_t)(r0 + r) * S.ld_x + (((e & (XVEC - 1)) ^ (r & SWZ)) << 2),
                                      xbig + (e0 << 2));
                        }
                    }
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                    lds_barrier();
                    for (int mb = 0; mb < ((rows + 15) >> 4); ++mb) {
                        const int arow = min(16 * mb + col, rows - 1);
                        const float* xrow = xbig + arow * NX;
                        mfma4 acc0 = {bv[h], bv[h], bv[h], bv[h]}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int s = 0; s < NX16; ++s) {
                            const float4 av = *reinterpret_cast<const float4*>(xrow + (((4 * s + g) ^ (arow & SWZ)) << 2));
                            acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(av.x, w[h][s][0], acc0, 0, 0, 0);
                            acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(av.y, w[h][s][1], acc1, 0, 0, 0);
                            acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(av.z, w[h][s][2], acc0, 0, 0, 0);
                            acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(av.w, w[h][s][3], acc1, 0, 0, 0);
                        }
                        const mfma4 r4 = acc0 + acc1;
                        const int row = r0 + 16 * mb + 4 * g;
                        float* tp = tile + ((unit_ch[h] * kx + row) << psh) + pcol;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            float* q = 16 * mb + 4 * g + i < rows ? tp + (i << psh) : sink;
                            *q = r4[i];
                        }
                    }
                    lds_barrier();      // the chunk may be replaced; after the last one: the piece's tile complete
                }
                // gather over the piece: a quarter of its columns per lane
                const int hsh = psh - 2;
                const int hr = tid >> hsh, hl = tid & ((1 << hsh) - 1);
                const char* tcol = reinterpret_cast<const char*>(tile) + 16 * hl;
                for (int r = hr; r < m; r += T >> hsh) {
                    const int p0 = rp[r], p1 = rp[r + 1];
                    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
                    for (int p = p0; p < p1; p += 4) {
                        int c[4];
                        float v[4];
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const int idx = min(p + t, p1 - 1);
                            c[t] = cols[idx];
                            v[t] = p + t < p1 ? vals[idx] : 0.f;
                        }
                        float4 bq[4];
#pragma unroll
                        for (int t = 0; t < 4; ++t) bq[t] = *reinterpret_cast<const float4*>(tcol + (c[t] << (psh + 2)));
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            acc.x = fmaf(v[t], bq[t].x, acc.x);
                            acc.y = fmaf(v[t], bq[t].y, acc.y);
                            acc.z = fmaf(v[t], bq[t].z, acc.z);
                            acc.w = fmaf(v[t], bq[t].w, acc.w);
                        }
                    }
                    float* yp = y + (bg.out_row + r) * S.ld_y + f0 + (h << psh) + 4 * hl;
                    if (S.accumulate) {
                        const float4 old = *reinterpret_cast<const float4*>(yp);
                        acc.x += old.x, acc.y += old.y, acc.z += old.z, acc.w += old.w;
                    }
                    store_out<4>(yp, acc);
                }
                lds_barrier();          // the piece's tile may be overwritten
            }
        }
        if (jn >= j1) return;
    }

    // the records of this graph and the next sit in scalar registers; the one after that is
    // fetched a trip ahead
    const int jbase = jn;
    StreamSet cur = sets[jn];
    StreamSet nxt = sets[min(jn + 1, j1 - 1)];
    request(cur, 0);
    for (int j = jn; j < j1; ++j) {
        const int b = (j - jbase) & 1;
        const StreamSet ahead = sets[min(j + 2, j1 - 1)];
        const int kx = cur.kx;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wavefront's requests for graph j
        lds_barrier();                                     // everyone's; everyone is done with graph j - 1
        store_pending();
        if (j + 1 < j1) request(nxt, b ^ 1);

        // The CSR block of this graph arrived a trip ago: the entry range of this lane's first
        // output row and its first four entries are read now, so that after the matrix phase
        // the gather starts with the tile reads instead of two more dependent LDS round trips.
        const int m = cur.m;
        const int* rp = cbase + b * S.csr_words;
        const int* cols = rp + ((m + 4) & ~3);
        const float* vals = reinterpret_cast<const float*>(cols + ((cur.nnz + 3) & ~3));
        int first_p0 = 0, first_p1 = 0;
        int fc[4] = {0, 0, 0, 0};
        float fv[4] = {0.f, 0.f, 0.f, 0.f};
        if (r_lane < m) {
            first_p0 = rp[r_lane];
            first_p1 = rp[r_lane + 1];
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (first_p0 + t < first_p1) {
                    fc[t] = cols[first_p0 + t];
                    fv[t] = vals[first_p0 + t];
                }
        }

        // ---- dense tile: [X_i W[0] + bias[0]; ...; X_i W[M-1] + bias[M-1]] -> LDS
        // With lists of the rows in use (S.compact) a wavefront makes only the rows of its
        // channel's tile that an entry of that channel names: block mb holds the rows
        // lst[16 mb ..] of X_i and goes to tile rows trow0 + 16 mb ..; without, all kx rows.
        const float* xs = xbase + b * S.x_words;
        int rows_w = kx, trow0[U];
        const int* lst = nullptr;
#pragma unroll
        for (int u = 0; u < U; ++u) trow0[u] = unit_ch[u] * kx;
        if (S.compact) {
            const int* cnt = reinterpret_cast<const int*>(vals + ((cur.nnz + 3) & ~3));
            const int c4 = (S.channels + 3) & ~3;
            rows_w = cnt[unit_ch[0]];
#pragma unroll
            for (int u = 0; u < U; ++u) trow0[u] = cnt[c4 + unit_ch[u]];
            lst = cnt + 2 * c4 + unit_ch[0] * kx;
        }
        const int nmb = (rows_w + 15) >> 4;
        auto x_row = [&](int i) {       // the row of X_i that is row i of this wavefront's blocks
            const int r = min(i, rows_w - 1);
            return S.compact ? (r >= 0 ? lst[r] : 0) : r;
        };
        float4 a[NX16];
        {
            const int arow = x_row(col);
            const float* xrow = xs + arow * NX;
#pragma unroll
            for (int s = 0; s < NX16; ++s)
                a[s] = *reinterpret_cast<const float4*>(xrow + (((4 * s + g) ^ (arow & SWZ)) << 2));
        }
        for (int mb = 0; mb < nmb; ++mb) {
            float4 an[NX16];
            {   // the next block's rows before this block's instructions (rows past the end repeat the last)
                const int arow = x_row(16 * (mb + 1) + col);
                const float* xrow = xs + arow * NX;
#pragma unroll
                for (int s = 0; s < NX16; ++s)
                    an[s] = *reinterpret_cast<const float4*>(xrow + (((4 * s + g) ^ (arow & SWZ)) << 2));
            }
            mfma4 acc[U][C];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int c = 0; c < C; ++c)
                    acc[u][c] = c == 0 ? mfma4{bv[u], bv[u], bv[u], bv[u]} : mfma4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < NX16; ++s) {
                const float ak[4] = {a[s].x, a[s].y, a[s].z, a[s].w};
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int u = 0; u < U; ++u)
                        acc[u][k % C] = __builtin_amdgcn_mfma_f32_16x16x4f32(ak[k], w[u][s][k], acc[u][k % C], 0, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                mfma4 r = acc[u][0];
                if (C == 2) r = r + acc[u][C - 1];
                float* tp = tile + ((trow0[u] + 16 * mb + 4 * g) << fsh) + unit_col[u];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float* q = 16 * mb + 4 * g + i < rows_w ? tp + (i << fsh) : sink;
                    *q = r[i];
                }
            }
#pragma unroll
            for (int s = 0; s < NX16; ++s) a[s] = an[s];
        }
        lds_barrier();                                     // tile complete

        // ---- gather over the merged CSR: Y_i = sum_ch A_i^ch tile_ch, into registers
        const char* tcol = reinterpret_cast<const char*>(tile) + 16 * l;
        const int lsh = fsh + 2;
        auto add4 = [&](float4& acc, const int (&c)[4], const float (&v)[4]) {
            float4 bq[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) bq[t] = *reinterpret_cast<const float4*>(tcol + (c[t] << lsh));
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                acc.x = fmaf(v[t], bq[t].x, acc.x);
                acc.y = fmaf(v[t], bq[t].y, acc.y);
                acc.z = fmaf(v[t], bq[t].z, acc.z);
                acc.w = fmaf(v[t], bq[t].w, acc.w);
            }
        };
        auto rest_of_row = [&](float4& acc, int p0, int p1) {     // four entries a trip, the tail masked
            for (int p = p0; p < p1; p += 4) {
                int c[4];
                float v[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int idx = min(p + t, p1 - 1);
                    c[t] = cols[idx];
                    v[t] = p + t < p1 ? vals[idx] : 0.f;
                }
                add4(acc, c, v);
            }
        };
        {
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            if (r_lane < m) {
                if (first_p0 < first_p1) add4(acc, fc, fv);
                rest_of_row(acc, first_p0 + 4, first_p1);
            }
            yv[0] = acc;
        }
#pragma unroll
        for (int q = 1; q < kStreamPasses; ++q) {
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            const int r = q * rows_per_pass + r_lane;
            if (q * rows_per_pass < m && r < m) rest_of_row(acc, rp[r], rp[r + 1]);
            yv[q] = acc;
        }
        pend_m = m;
        pend_row = cur.out_row;
        cur = nxt;
        nxt = ahead;
    }
    store_pending();
}

// ---------------------------------------------------------------------------------------
// Direct product for COO / SparseTensor operands (Fig. 3 with the output staged on chip as in
// Fig. 5(a,b)), in two forms per item (item.mode):
//  * sorted: the workgroup counts the operation's entries per output row (integer LDS atomics),
//    scans the counts, scatters (dense row, value) pairs into row order in LDS and sums each row
//    in registers, a lane group per row: no floating-point atomics and no output tile.  The
//    dense tile sits in LDS beside the pairs where the scheduler found room; otherwise the dense
//    rows are read from memory, eight in flight per group.
//  * the paper's form: the item's output tile lives in LDS; a group of L lanes takes one stored
//    entry at a time (L = the tile's vectors per row rounded up to a power of two, at most 64),
//    reads the dense row it names and adds value * row into the tile with LDS floating-point
//    atomics; the tile is then streamed out.  Four entries per group are in flight at once.
//    What the paper reads from global memory entry by entry - the index pairs, the values and
//    the dense rows - is first copied to LDS in bulk where the scheduler found room: a
//    workgroup then pays one round trip to memory instead of one per entry.
// Entries outside the item's row range (or outside the matrix) are skipped.
// ---------------------------------------------------------------------------------------
template <int VEC>
__global__ void __launch_bounds__(kThreads)
bspmm_coo_kernel(const CooLaunchParams P)
{
    extern __shared__ __align__(16) float tile[];
    using V = typename Vec<VEC>::type;
    const CooItem it = P.items[blockIdx.x];
    const int tid = threadIdx.x;
    const int stride = round_up(it.fw, 4);
    const int nvec = (it.fw + VEC - 1) / VEC;          // VEC == 4 implies fw % 4 == 0
    const bool st_b = (it.mode & 1) != 0, st_e = (it.mode & 2) != 0;
    const bool sorted = (it.mode & 4) != 0 && st_e;
    float* bt = sorted ? tile : tile + it.nrows * stride;
    int2* ent = reinterpret_cast<int2*>(bt + (st_b ? it.k * stride : 0));
    float* ev = reinterpret_cast<float*>(ent + it.nnz);

    const int log2L = ilog2(min(64, pow2_ceil(nvec)));
    const int L = 1 << log2L;
    const int lane = tid & (L - 1);
    const int grp = tid >> log2L;
    const int G = kThreads >> log2L;
    const int32_t* __restrict__ id = P.ids + 2 * it.nz_off;
    const float* __restrict__ va = P.values + it.nz_off;
    const int sel = P.transposed ? 1 : 0;
    const float* __restrict__ in = P.in + it.in_row_off * P.ld_in + it.f0;

    // Items the host marked so (mode bit 2) sort their entries by output row on chip - count
    // per row, scan, scatter of (dense row, value) pairs into row order - and then run the row
    // gather of the CSR kernels over them: no floating-point atomics and no output tile, a
    // row's sum is kept in registers and stored once.  The pairs take the place of the staged
    // entries; behind them sit the row counts and the row pointers.
    int2* sp = ent;
    int* s_cnt = reinterpret_cast<int*>(sp + it.nnz);
    int* s_rp = s_cnt + it.nrows + 1;

    // ---- staging: every load is issued before anything is waited for
    bool direct = false;
    if (st_b) {
        direct = VEC == 4 && (nvec & (nvec - 1)) == 0;      // then stride == fw: rows are packed
        if (direct) {
            const int sh = ilog2(nvec);
            const int total = it.k << sh;                    // float4 in the tile
            const int wl = tid & 63;
            for (int e0 = (tid >> 6) << 6; e0 < total; e0 += kThreads) {
                const int e = e0 + wl;
                if (e < total) {
                    const float* gp = in + (int64_t)(e >> sh) * P.ld_in + ((e & (nvec - 1)) << 2);
                    __builtin_amdgcn_global_load_lds(
                        (const void __attribute__((address_space(1)))*)gp,
                        (void __attribute__((address_space(3)))*)(bt + (e0 << 2)), 16, 0, 0);
                }
            }
        } else {
            for (int r0 = grp; r0 < it.k; r0 += 4 * G)
                for (int j = lane; j < nvec; j += L) {
                    V t[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (r0 + u * G < it.k)
                            t[u] = load_vec<VEC>(in + (int64_t)(r0 + u * G) * P.ld_in + j * VEC);
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (r0 + u * G < it.k) store_vec<VEC>(bt + (r0 + u * G) * stride + j * VEC, t[u]);
                }
        }
    }
    if (sorted) {
        __shared__ int wave_sum[kThreads / 64];
        __shared__ int carry;
        // The first four entries of every lane stay in registers between the count and the
        // scatter; what lies beyond them is read again.
        constexpr int KEEP = 4;
        int kr[KEEP], kc[KEEP];
        float kv[KEEP];
        auto entry = [&](int p, int& r, int& c, float& v) {
            r = id[2 * p + sel] - it.row0;
            c = id[2 * p + 1 - sel];
            v = va[p];
        };
#pragma unroll
        for (int u = 0; u < KEEP; ++u) {
            const int p = tid + u * kThreads;
            kr[u] = -1;
            kc[u] = 0;
            kv[u] = 0.f;
            if (p < it.nnz) entry(p, kr[u], kc[u], kv[u]);
        }
        for (int i = tid; i <= it.nrows; i += kThreads) s_cnt[i] = 0;
        lds_barrier();
#pragma unroll
        for (int u = 0; u < KEEP; ++u) {
            if (!((unsigned)kr[u] < (unsigned)it.nrows && (unsigned)kc[u] < (unsigned)it.k)) kr[u] = -1;
            if (kr[u] >= 0) atomicAdd(&s_cnt[kr[u]], 1);
        }
        for (int p = tid + KEEP * kThreads; p < it.nnz; p += kThreads) {
            int r, c;
            float v;
            entry(p, r, c, v);
            if ((unsigned)r < (unsigned)it.nrows && (unsigned)c < (unsigned)it.k) atomicAdd(&s_cnt[r], 1);
        }
        if (tid == 0) carry = 0;
        lds_barrier();
        // exclusive scan over the rows, 256 at a time (the counts are cleared for the scatter)
        const int wv = tid >> 6, wlane = tid & 63;
        for (int base = 0; base < it.nrows; base += kThreads) {
            const int i = base + tid;
            const int c = i < it.nrows ? s_cnt[i] : 0;
            int x = c;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int y = __shfl_up(x, off);
                if (wlane >= off) x += y;
            }
            if (wlane == 63) wave_sum[wv] = x;
            lds_barrier();
            int before = carry;
            for (int q = 0; q < wv; ++q) before += wave_sum[q];
            if (i < it.nrows) {
                s_rp[i] = before + x - c;
                s_cnt[i] = 0;
            }
            lds_barrier();
            if (tid == kThreads - 1) carry = before + x;
            lds_barrier();
        }
        if (tid == 0) s_rp[it.nrows] = carry;
        // (dense row, value) pairs in row order (inside a row: the order the lanes get there)
#pragma unroll
        for (int u = 0; u < KEEP; ++u)
            if (kr[u] >= 0)
                sp[s_rp[kr[u]] + atomicAdd(&s_cnt[kr[u]], 1)] =
                    make_int2(st_b ? kc[u] * stride : kc[u], __float_as_int(kv[u]));
        for (int p = tid + KEEP * kThreads; p < it.nnz; p += kThreads) {
            int r, c;
            float v;
            entry(p, r, c, v);
            if ((unsigned)r < (unsigned)it.nrows && (unsigned)c < (unsigned)it.k)
                sp[s_rp[r] + atomicAdd(&s_cnt[r], 1)] = make_int2(st_b ? c * stride : c, __float_as_int(v));
        }
        if (direct) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // direct-to-LDS loads landed
        __syncthreads();
        // row gather: one lane group per output row; four entries in flight from LDS, eight
        // from memory
        float* outp = P.out + (it.out_row_off + it.row0) * P.ld_out + it.f0;
        auto gather = [&](auto width) {
            constexpr int W = decltype(width)::value;
            for (int rr = grp; rr < it.nrows; rr += G) {
                const int q0 = s_rp[rr], q1 = s_rp[rr + 1];
                for (int j = lane; j < nvec; j += L) {
                    V acc = Vec<VEC>::zero();
                    for (int q = q0; q < q1; q += W) {
                        int2 e[W];
#pragma unroll
                        for (int u = 0; u < W; ++u) e[u] = sp[min(q + u, q1 - 1)];
                        V b[W];
#pragma unroll
                        for (int u = 0; u < W; ++u)
                            b[u] = st_b ? load_vec<VEC>(bt + e[u].x + j * VEC)
                                        : load_vec<VEC>(in + (int64_t)e[u].x * P.ld_in + j * VEC);
#pragma unroll
                        for (int u = 0; u < W; ++u) {
                            const float v = q + u < q1 ? __int_as_float(e[u].y) : 0.f;
                            float* af = reinterpret_cast<float*>(&acc);
                            const float* bf = reinterpret_cast<const float*>(&b[u]);
#pragma unroll
                            for (int c = 0; c < VEC; ++c) af[c] = fmaf(v, bf[c], af[c]);
                        }
                    }
                    store_out<VEC>(outp + (int64_t)rr * P.ld_out + j * VEC, acc);
                }
            }
        };
        if (st_b) gather(std::integral_constant<int, 4>{});
        else gather(std::integral_constant<int, 8>{});
        return;
    }

    if (st_e) {
        for (int p0 = tid; p0 < it.nnz; p0 += 2 * kThreads) {
            int r[2], c[2];
            float v[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int p = p0 + u * kThreads;
                if (p < it.nnz) {
                    r[u] = id[2 * p + sel] - it.row0;
                    c[u] = id[2 * p + 1 - sel];
                    v[u] = va[p];
                }
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int p = p0 + u * kThreads;
                if (p < it.nnz) {
                    const bool ok = (unsigned)r[u] < (unsigned)it.nrows && (unsigned)c[u] < (unsigned)it.k;
                    ent[p] = make_int2(ok ? r[u] * stride : -1, st_b ? c[u] * stride : c[u]);
                    ev[p] = v[u];
                }
            }
        }
    }
    {
        float4* t4 = reinterpret_cast<float4*>(tile);
        const int n4 = it.nrows * (stride >> 2);
        for (int i = tid; i < n4; i += kThreads) t4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if (direct) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // direct-to-LDS loads landed
    __syncthreads();

    // ---- one lane group per entry
    constexpr int U = 4;
    for (int p0 = grp; p0 < it.nnz; p0 += U * G) {
        int ro[U], co[U];
        float v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int p = p0 + u * G;
            ro[u] = -1;
            co[u] = 0;
            v[u] = 0.f;
            if (p < it.nnz) {
                if (st_e) {
                    const int2 e = ent[p];
                    ro[u] = e.x;
                    co[u] = e.y;
                    v[u] = ev[p];
                } else {
                    const int r = id[2 * p + sel] - it.row0;
                    const int c = id[2 * p + 1 - sel];
                    v[u] = va[p];
                    if ((unsigned)r < (unsigned)it.nrows && (unsigned)c < (unsigned)it.k) {
                        ro[u] = r * stride;
                        co[u] = c;             // mode bit 0 is never set without bit 1
                    }
                }
            }
        }
        for (int j = lane; j < nvec; j += L) {
            V b[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (ro[u] >= 0)
                    b[u] = st_b ? load_vec<VEC>(bt + co[u] + j * VEC)
                                : load_vec<VEC>(in + (int64_t)co[u] * P.ld_in + j * VEC);
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (ro[u] >= 0) {
                    float* dst = tile + ro[u] + j * VEC;
                    const float* bf = reinterpret_cast<const float*>(&b[u]);
#pragma unroll
                    for (int e = 0; e < VEC; ++e)
                        __hip_atomic_fetch_add(dst + e, v[u] * bf[e], __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_WORKGROUP);
                }
        }
    }
    __syncthreads();

    float* out = P.out + (it.out_row_off + it.row0) * P.ld_out + it.f0;
    for (int rr = grp; rr < it.nrows; rr += G)
        for (int j = lane; j < nvec; j += L)
            store_out<VEC>(out + (int64_t)rr * P.ld_out + j * VEC,
                           load_vec<VEC>(tile + rr * stride + j * VEC));
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
using KernelFn = void (*)(const LaunchParams);

static KernelFn kernel_variant(bool vec4, bool slices, bool hubs, bool merged = false)
{
    static const KernelFn table[16] = {
        bspmm_kernel<1, false, false>, bspmm_kernel<1, false, true>,
        bspmm_kernel<1, true, false>,  bspmm_kernel<1, true, true>,
        bspmm_kernel<4, false, false>, bspmm_kernel<4, false, true>,
        bspmm_kernel<4, true, false>,  bspmm_kernel<4, true, true>,
        bspmm_kernel<1, false, false, true>, bspmm_kernel<1, false, true, true>,
        bspmm_kernel<1, true, false, true>,  bspmm_kernel<1, true, true, true>,
        bspmm_kernel<4, false, false, true>, bspmm_kernel<4, false, true, true>,
        bspmm_kernel<4, true, false, true>,  bspmm_kernel<4, true, true, true>};
    return table[(merged ? 8 : 0) + (vec4 ? 4 : 0) + (slices ? 2 : 0) + (hubs ? 1 : 0)];
}

// Workgroups of bspmm_kernel the current device holds at once (0 if it cannot be asked).
int bspmm_max_resident_workgroups(int lds_bytes, bool slices, bool hubs)
{
    int per_cu4 = 0, per_cu1 = 0, dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess)
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu4, kernel_variant(true, slices, hubs),
                                                         kThreads, (size_t)lds_bytes);
    if (e == hipSuccess)
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu1, kernel_variant(false, slices, hubs),
                                                         kThreads, (size_t)lds_bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    const int per_cu = per_cu4 < per_cu1 ? per_cu4 : per_cu1;
    return per_cu > 0 && cus > 0 ? per_cu * cus : 0;
}

// Registers, LDS and occupancy of kernel `which` (BSPMM_KERNEL_* of the public header) on the
// current device.  out: vgprs, sgprs, static LDS, scratch, lanes per workgroup, workgroups per CU
// at `lds_bytes` of dynamic LDS, compute units.
hipError_t kernel_resources(int which, int lds_bytes, int out[7])
{
    const void* fn = nullptr;
    int threads = kThreads;
    switch (which) {
        case 0: fn = reinterpret_cast<const void*>(&bspmm_lean_kernel); break;
        case 1: fn = reinterpret_cast<const void*>(&bspmm_kernel<4, false, false, false>); break;
        case 2: fn = reinterpret_cast<const void*>(&bspmm_kernel<1, false, false, false>); break;
        case 3: fn = reinterpret_cast<const void*>(&bspmm_gcn_kernel<false, false>); break;
        case 4: fn = reinterpret_cast<const void*>(&bspmm_gcn_kernel<false, true>); break;
        case 5: fn = reinterpret_cast<const void*>(&build_sorted_kernel<false, kThreads>); break;
        case 6:
            fn = reinterpret_cast<const void*>(&build_sorted_kernel<false, kBuildThreadsLarge>);
            threads = kBuildThreadsLarge;
            break;
        case 7: fn = reinterpret_cast<const void*>(&bspmm_coo_kernel<4>); break;
        case 8: fn = reinterpret_cast<const void*>(&bspmm_gcn_stream_kernel<4, 2, 4>); break;
        default: return hipErrorInvalidValue;
    }
    hipFuncAttributes a;
    hipError_t e = hipFuncGetAttributes(&a, fn);
    if (e != hipSuccess) return e;
    int per_cu = 0, dev = 0, cus = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, threads, (size_t)lds_bytes);
    if (e == hipSuccess) e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    out[0] = a.numRegs;
    out[1] = 0;
    out[2] = (int)a.sharedSizeBytes;
    out[3] = (int)a.localSizeBytes;
    out[4] = threads;
    out[5] = per_cu;
    out[6] = cus;
    return hipSuccess;
}

hipError_t launch_bspmm(const LaunchParams& P, int grid, int lds_bytes, bool vec4, bool slices,
                        bool hubs, bool merged, hipStream_t stream)
{
    if (grid <= 0) return hipSuccess;
    hipLaunchKernelGGL(kernel_variant(vec4, slices, hubs, merged), dim3(grid), dim3(kThreads),
                       lds_bytes, stream, P);
    return hipGetLastError();
}

hipError_t launch_bspmm_lean(const LeanItem* items, const LaunchParams& P, int grid, int lds_bytes,
                             hipStream_t stream)
{
    if (grid <= 0) return hipSuccess;
    hipLaunchKernelGGL(bspmm_lean_kernel, dim3(grid), dim3(kThreads), lds_bytes, stream, items,
                       P.rpt, P.colids, P.values, P.in, P.out, (uint32_t)P.ld_in,
                       (uint32_t)P.ld_out, (uint32_t)(lds_bytes / 4));
    return hipGetLastError();
}

hipError_t launch_lean_hints(LeanItem* items, int n, const int32_t* rpt, hipStream_t stream)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(lean_hints_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, items, n, rpt);
    return hipGetLastError();
}

using FrontFn = void (*)(const LaunchParams);

static FrontFn front_variant(bool accumulate, bool sets, bool wide)
{
    static const FrontFn table[8] = {
        bspmm_gcn_kernel<false, false>, bspmm_gcn_kernel<true, false>,
        bspmm_gcn_kernel<false, true>, bspmm_gcn_kernel<true, true>,
        bspmm_gcn_kernel<false, false, 2 * kThreads>, bspmm_gcn_kernel<true, false, 2 * kThreads>,
        bspmm_gcn_kernel<false, true, 2 * kThreads>, bspmm_gcn_kernel<true, true, 2 * kThreads>};
    return table[(wide ? 4 : 0) + (sets ? 2 : 0) + (accumulate ? 1 : 0)];
}

// Workgroups of the one-launch layer kernel one CU of the current device holds (0 if it cannot
// be asked); wide: workgroups of eight wavefronts.
int front_workgroups_per_cu(bool sets, bool wide, int lds_bytes)
{
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, front_variant(false, sets, wide),
                                                     wide ? 2 * kThreads : kThreads, (size_t)lds_bytes) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    return per_cu;
}

hipError_t launch_bspmm_gcn(const LaunchParams& P, int grid, int lds_bytes, bool accumulate,
                            bool sets, bool wide, hipStream_t stream)
{
    if (grid <= 0) return hipSuccess;
    hipLaunchKernelGGL(front_variant(accumulate, sets, wide), dim3(grid), dim3(wide ? 2 * kThreads : kThreads),
                       lds_bytes, stream, P);
    return hipGetLastError();
}

using StreamFn = void (*)(const StreamSet*, const int32_t*, const int32_t*, const float*, const float*,
                          const float*, float*, const StreamShape);

// (n_X / 16, blocks per wavefront, wavefronts) -> kernel; null for shapes the streaming kernel is
// not built for
static StreamFn stream_variant(int nx16, int units, int waves)
{
    if (waves == 4 && units == 1) {
        switch (nx16) {
        case 1: return bspmm_gcn_stream_kernel<1, 1, 4>;
        case 2: return bspmm_gcn_stream_kernel<2, 1, 4>;
        case 4: return bspmm_gcn_stream_kernel<4, 1, 4>;
        case 8: return bspmm_gcn_stream_kernel<8, 1, 4>;
        }
    } else if (waves == 4 && units == 2) {
        switch (nx16) {
        case 1: return bspmm_gcn_stream_kernel<1, 2, 4>;
        case 2: return bspmm_gcn_stream_kernel<2, 2, 4>;
        case 4: return bspmm_gcn_stream_kernel<4, 2, 4>;
        }
    } else if (waves == 8 && units == 2) {      // eight channels: a wavefront per channel
        switch (nx16) {
        case 1: return bspmm_gcn_stream_kernel<1, 2, 8>;
        case 2: return bspmm_gcn_stream_kernel<2, 2, 8>;
        case 4: return bspmm_gcn_stream_kernel<4, 2, 8>;
        }
    } else if (waves == 8 && units == 1) {      // the same on tiles of 16 columns (n_X = 128, F = 16, 48, ...)
        switch (nx16) {
        case 1: return bspmm_gcn_stream_kernel<1, 1, 8>;
        case 2: return bspmm_gcn_stream_kernel<2, 1, 8>;
        case 4: return bspmm_gcn_stream_kernel<4, 1, 8>;
        case 8: return bspmm_gcn_stream_kernel<8, 1, 8>;
        }
    }
    return nullptr;
}

bool stream_supported(int nx16, int units, int waves) { return stream_variant(nx16, units, waves) != nullptr; }

// Workgroups of the streaming kernel one CU of the current device holds (0 if it cannot be asked).
int stream_workgroups_per_cu(int nx16, int units, int waves, int lds_bytes)
{
    const StreamFn fn = stream_variant(nx16, units, waves);
    int per_cu = 0;
    if (!fn) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, 64 * waves, (size_t)lds_bytes) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    return per_cu;
}

hipError_t launch_bspmm_gcn_stream(const StreamParams& P, int nx16, int units, int waves, int grid,
                                   int lds_bytes, hipStream_t stream)
{
    if (grid <= 0) return hipSuccess;
    const StreamFn fn = stream_variant(nx16, units, waves);
    if (!fn) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fn, dim3(grid), dim3(64 * waves), lds_bytes, stream, P.sets, P.list, P.merged, P.x,
                       P.w, P.bias, P.y, P.shape);
    return hipGetLastError();
}

hipError_t launch_build_transpose(const OpRecord* ops, int batch, int threads, int lds_bytes,
                                  const int32_t* rpt, const int32_t* colids,
                                  const float* values, int32_t* rpt_t, int32_t* colids_t,
                                  float* values_t, int32_t* gscratch, const int32_t* order,
                                  hipStream_t stream)
{
    if (batch <= 0) return hipSuccess;
    if (threads == kBuildThreadsLarge)
        hipLaunchKernelGGL((build_sorted_kernel<false, kBuildThreadsLarge>), dim3(batch),
                           dim3(kBuildThreadsLarge), lds_bytes, stream, ops, rpt, colids, values,
                           rpt_t, colids_t, values_t, gscratch, order);
    else
        hipLaunchKernelGGL((build_sorted_kernel<false, kThreads>), dim3(batch), dim3(kThreads),
                           lds_bytes, stream, ops, rpt, colids, values, rpt_t, colids_t, values_t,
                           gscratch, order);
    return hipGetLastError();
}

hipError_t launch_merge_sets(const SetRecord* sets, int count, const int32_t* rpt,
                             const int32_t* colids, const float* values, int32_t* merged,
                             hipStream_t stream)
{
    if (count <= 0) return hipSuccess;
    hipLaunchKernelGGL(merge_sets_kernel, dim3(count), dim3(kThreads), 0, stream, sets, rpt, colids,
                       values, merged);
    return hipGetLastError();
}

hipError_t launch_bspmm_coo(const CooLaunchParams& P, int grid, int lds_bytes, bool vec4,
                            hipStream_t stream)
{
    if (grid <= 0) return hipSuccess;
    if (vec4)
        hipLaunchKernelGGL(bspmm_coo_kernel<4>, dim3(grid), dim3(kThreads), lds_bytes, stream, P);
    else
        hipLaunchKernelGGL(bspmm_coo_kernel<1>, dim3(grid), dim3(kThreads), lds_bytes, stream, P);
    return hipGetLastError();
}

// COO (index pairs `ids`, values) -> CSR arrays of every operation.
hipError_t launch_build_from_coo(const OpRecord* ops, int batch, int threads, int lds_bytes, const int32_t* ids,
                                 const float* values, int32_t* rpt, int32_t* colids,
                                 float* csr_values, int32_t* gscratch, const int32_t* order,
                                 hipStream_t stream)
{
    if (batch <= 0) return hipSuccess;
    if (threads == kBuildThreadsLarge)
        hipLaunchKernelGGL((build_sorted_kernel<true, kBuildThreadsLarge>), dim3(batch),
                           dim3(kBuildThreadsLarge), lds_bytes, stream, ops,
                           static_cast<const int32_t*>(nullptr), ids, values, rpt, colids,
                           csr_values, gscratch, order);
    else
        hipLaunchKernelGGL((build_sorted_kernel<true, kThreads>), dim3(batch), dim3(kThreads),
                           lds_bytes, stream, ops, static_cast<const int32_t*>(nullptr), ids,
                           values, rpt, colids, csr_values, gscratch, order);
    return hipGetLastError();
}

hipError_t launch_validate_coo(const OpRecord* ops, int batch, const int32_t* ids, int32_t* flag,
                               hipStream_t stream)
{
    hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(64), 0, stream, flag, 0x7fffffff, 1);
    if (batch > 0)
        hipLaunchKernelGGL(validate_coo_kernel, dim3(batch), dim3(kThreads), 0, stream, ops, ids, flag);
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
