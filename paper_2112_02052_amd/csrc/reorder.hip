// Row clustering before SGT, and the symmetric permutation of a CSR pattern.
//
// The paper's related-work section calls row reordering orthogonal and complementary to SGT and names
// no algorithm.  SGT pays off when the rows of a window share neighbours; a labelling that scatters the
// members of a community over the whole id range (the randomly relabelled clustered workload) destroys
// that.  This pass is a cheap, deterministic way to get it back:
//   1. hash(v) = splitmix64 of (seed, v); nodes are compared by (hash, id);
//   2. parent(v) = the smallest node of {v} + N(v);
//   3. root(v)   = the fixed point of v -> parent(v) (hashes fall along the chain, so it ends);
//   4. label = root, then `refine` synchronous rounds of "take the most frequent label among the first
//      128 stored neighbours" (ties to the smallest label id; rows without entries keep theirs);
//   5. perm = the nodes sorted by (label, parent, id) -- two stable radix sorts.
// Nodes that share neighbours tend to share the smallest neighbour, so they land in the same tree and
// next to each other.  Every step is a streaming pass over the edge list or the node list; the hash is
// computed from the id, so step 2 gathers nothing.
#include "common.h"

namespace tcg {

namespace {

constexpr int kThreads = 256;
constexpr int kGroup = 16;                 // lanes per row
constexpr int kRefineMax = 128;            // neighbours looked at by a refinement round
constexpr int kLongRow = 4096;             // rows above this length get a whole workgroup in step 2

__device__ __forceinline__ uint64_t node_hash(uint64_t seed, int32_t v)
{
    uint64_t z = seed + ((uint64_t)(uint32_t)v + 1ull) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// (hash, id) order
__device__ __forceinline__ bool node_less(uint64_t ha, int32_t a, uint64_t hb, int32_t b)
{
    return ha < hb || (ha == hb && a < b);
}

// flag bit 0 = row_ptr ends wrong, bit 1 = row_ptr not monotone, bit 2 = column outside [0, n)
__global__ void check_square_kernel(int32_t n, int64_t nnz, const int32_t *__restrict__ rp,
                                    const int32_t *__restrict__ ci, int *flag)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int bad = 0;
    if (i == 0 && (rp[0] != 0 || (int64_t)rp[n] != nnz)) bad |= 1;
    for (int64_t r = i; r < n; r += stride)
        if (rp[r] > rp[r + 1] || rp[r] < 0) bad |= 2;
    if (bad == 0)       // the columns are only read once the row pointers of this thread's share are sane
        for (int64_t e = i; e < nnz; e += stride)
            if (ci[e] < 0 || ci[e] >= n) bad |= 4;
    if (bad) atomicOr(flag, bad);
}

// Step 2 for rows of at most kLongRow entries: kGroup lanes per row.  Longer rows are appended to
// long_rows (their order does not matter: each row writes only its own parent).
__global__ __launch_bounds__(kThreads) void parent_kernel(int32_t n, const int32_t *__restrict__ rp,
                                                          const int32_t *__restrict__ ci, uint64_t seed,
                                                          int32_t *__restrict__ parent,
                                                          int32_t *__restrict__ long_rows, int32_t *n_long)
{
    const int lane = threadIdx.x % kGroup;
    const int64_t v = ((int64_t)blockIdx.x * kThreads + threadIdx.x) / kGroup;
    if (v >= n) return;                      // kGroup divides the wavefront: whole groups leave together
    const int32_t b = rp[v], e = rp[v + 1];
    if (e - b > kLongRow) {
        if (lane == 0) long_rows[atomicAdd(n_long, 1)] = (int32_t)v;
        return;
    }
    int32_t best = (int32_t)v;
    uint64_t hbest = node_hash(seed, best);
    for (int32_t k = b + lane; k < e; k += kGroup) {
        const int32_t u = ci[k];
        const uint64_t hu = node_hash(seed, u);
        if (node_less(hu, u, hbest, best)) { hbest = hu; best = u; }
    }
#pragma unroll
    for (int off = 1; off < kGroup; off <<= 1) {
        const int32_t ob = __shfl_xor(best, off, kGroup);
        const uint64_t oh = ((uint64_t)(uint32_t)__shfl_xor((int)(hbest >> 32), off, kGroup) << 32) |
                            (uint32_t)__shfl_xor((int)(uint32_t)hbest, off, kGroup);
        if (node_less(oh, ob, hbest, best)) { hbest = oh; best = ob; }
    }
    if (lane == 0) parent[v] = best;
}

// Step 2 for the long rows: one workgroup per row.  Launched with an upper bound of the count.
__global__ __launch_bounds__(kThreads) void parent_long_kernel(const int32_t *__restrict__ rp,
                                                               const int32_t *__restrict__ ci, uint64_t seed,
                                                               int32_t *__restrict__ parent,
                                                               const int32_t *__restrict__ long_rows,
                                                               const int32_t *__restrict__ n_long)
{
    __shared__ uint64_t s_h[kThreads];
    __shared__ int32_t s_v[kThreads];
    if ((int32_t)blockIdx.x >= *n_long) return;
    const int32_t v = long_rows[blockIdx.x];
    int32_t best = v;
    uint64_t hbest = node_hash(seed, best);
    for (int32_t k = rp[v] + threadIdx.x; k < rp[v + 1]; k += kThreads) {
        const int32_t u = ci[k];
        const uint64_t hu = node_hash(seed, u);
        if (node_less(hu, u, hbest, best)) { hbest = hu; best = u; }
    }
    s_h[threadIdx.x] = hbest;
    s_v[threadIdx.x] = best;
    __syncthreads();
    for (int off = kThreads / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off && node_less(s_h[threadIdx.x + off], s_v[threadIdx.x + off], s_h[threadIdx.x], s_v[threadIdx.x])) {
            s_h[threadIdx.x] = s_h[threadIdx.x + off];
            s_v[threadIdx.x] = s_v[threadIdx.x + off];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) parent[v] = s_v[0];
}

// Step 3.  The chain from v visits nodes of strictly decreasing (hash, id), so it ends at a node that
// is its own parent.
__global__ void root_kernel(int32_t n, const int32_t *__restrict__ parent, int32_t *__restrict__ label)
{
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= n) return;
    int32_t p = (int32_t)v, q = parent[p];
    while (q != p) {
        p = q;
        q = parent[p];
    }
    label[v] = p;
}

// Step 4, one round: kGroup lanes per row; the labels of the row's first kRefineMax neighbours are
// staged in LDS and every lane counts, for its share of them, how often that label occurs.
__global__ __launch_bounds__(kThreads) void refine_kernel(int32_t n, const int32_t *__restrict__ rp,
                                                          const int32_t *__restrict__ ci,
                                                          const int32_t *__restrict__ label_in,
                                                          int32_t *__restrict__ label_out)
{
    __shared__ int32_t s_lab[kThreads / kGroup][kRefineMax + 1];   // + 1: the groups of a wavefront read different banks
    const int lane = threadIdx.x % kGroup, grp = threadIdx.x / kGroup;
    const int64_t v = (int64_t)blockIdx.x * (kThreads / kGroup) + grp;
    const bool live = v < n;
    const int32_t b = live ? rp[v] : 0;
    const int32_t k = live ? min(rp[v + 1] - b, kRefineMax) : 0;
    for (int i = lane; i < k; i += kGroup) s_lab[grp][i] = label_in[ci[b + i]];
    __syncthreads();
    if (!live) return;
    int best_cnt = 0;
    int32_t best_lab = INT32_MAX;
    for (int i = lane; i < k; i += kGroup) {
        const int32_t li = s_lab[grp][i];
        int c = 0;
        for (int j = 0; j < k; ++j) c += s_lab[grp][j] == li;
        if (c > best_cnt || (c == best_cnt && li < best_lab)) { best_cnt = c; best_lab = li; }
    }
#pragma unroll
    for (int off = 1; off < kGroup; off <<= 1) {
        const int oc = __shfl_xor(best_cnt, off, kGroup);
        const int32_t ol = __shfl_xor(best_lab, off, kGroup);
        if (oc > best_cnt || (oc == best_cnt && ol < best_lab)) { best_cnt = oc; best_lab = ol; }
    }
    if (lane == 0) label_out[v] = k > 0 ? best_lab : label_in[v];
}

__global__ void gather_i32_kernel(int64_t n, const int32_t *__restrict__ idx, const int32_t *__restrict__ in,
                                  int32_t *__restrict__ out)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = in[idx[i]];
}

__global__ void fill_kernel(int32_t *p, int64_t n, int32_t v)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// inv[perm[i]] = i, and the new row lengths; flag bit 0 = entry outside [0, n), bit 1 = repeated entry.
__global__ void invert_perm_kernel(int32_t n, const int32_t *__restrict__ perm, const int32_t *__restrict__ rp,
                                   int32_t *__restrict__ inv, int32_t *__restrict__ deg, int *flag)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t o = perm[i];
    if (o < 0 || o >= n) {
        atomicOr(flag, 1);
        deg[i] = 0;
        return;
    }
    if (atomicCAS(&inv[o], -1, (int32_t)i) != -1) atomicOr(flag, 2);
    deg[i] = rp[o + 1] - rp[o];
}

// One thread per entry of the result: its row by bisection in the new row pointers.
__global__ void permute_entries_kernel(int32_t n, int64_t nnz, const int32_t *__restrict__ rp,
                                       const int32_t *__restrict__ ci, const int32_t *__restrict__ perm,
                                       const int32_t *__restrict__ inv, const int32_t *__restrict__ new_rp,
                                       int32_t *__restrict__ new_ci, int32_t *__restrict__ edge_perm)
{
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= nnz) return;
    int32_t lo = 0, hi = n;                  // last row i with new_rp[i] <= k
    while (hi - lo > 1) {
        const int32_t mid = lo + (hi - lo) / 2;
        if (new_rp[mid] <= k) lo = mid; else hi = mid;
    }
    const int32_t src = rp[perm[lo]] + (int32_t)(k - new_rp[lo]);
    new_ci[k] = inv[ci[src]];
    if (edge_perm) edge_perm[k] = src;
}

__global__ void set_last_kernel(int32_t *p, int64_t idx, int32_t v) { p[idx] = v; }

inline unsigned blocks_for(int64_t n, int per_block = 256) { return (unsigned)ceil_div(n > 0 ? n : 1, per_block); }

int bits_for(int64_t range)
{
    int bits = 1;
    while (bits < 31 && (1ll << bits) < range) ++bits;
    return bits;
}

}  // namespace

int reorder_rows_impl(int32_t n, int64_t nnz, const int32_t *d_row_ptr, const int32_t *d_col_idx, uint64_t seed,
                      int32_t refine, int32_t *d_perm, hipStream_t s)
{
    if (n == 0) return TCG_OK;
    if (radix_sort_scratch_bytes(n) == 0) return TCG_ERANGE;
    const size_t arr = ((size_t)n * 4 + 255) & ~(size_t)255;
    const int64_t max_long = nnz / kLongRow + 1;
    const size_t long_bytes = ((size_t)max_long * 4 + 255) & ~(size_t)255;
    // parent, label a/b, sorted keys, values of the first sort, long-row list, counters, sort scratch
    PoolBuf buf;
    buf.s = s;
    TCG_TRY(pool_alloc(&buf.p, 6 * arr + long_bytes + 256 + radix_sort_scratch_bytes(n)));
    char *base = static_cast<char *>(buf.p);
    int32_t *parent = reinterpret_cast<int32_t *>(base);
    int32_t *label_a = reinterpret_cast<int32_t *>(base + arr);
    int32_t *label_b = reinterpret_cast<int32_t *>(base + 2 * arr);
    int32_t *keys = reinterpret_cast<int32_t *>(base + 3 * arr);
    int32_t *order1 = reinterpret_cast<int32_t *>(base + 4 * arr);
    int32_t *keys2 = reinterpret_cast<int32_t *>(base + 5 * arr);
    int32_t *long_rows = reinterpret_cast<int32_t *>(base + 6 * arr);
    int32_t *counters = reinterpret_cast<int32_t *>(base + 6 * arr + long_bytes);   // [0] flag, [1] n_long
    void *sort_scratch = base + 6 * arr + long_bytes + 256;

    hipLaunchKernelGGL(fill_kernel, dim3(1), dim3(64), 0, s, counters, (int64_t)2, 0);
    hipLaunchKernelGGL(check_square_kernel, dim3((unsigned)std::min<int64_t>(ceil_div(std::max<int64_t>(nnz, n + 1), 256), 8192)),
                       dim3(256), 0, s, n, nnz, d_row_ptr, d_col_idx, counters);
    TCG_TRY(launch_status("check_square_kernel"));
    int h_flag = 0;
    TCG_HIP(hipMemcpyAsync(&h_flag, counters, sizeof(int), hipMemcpyDeviceToHost, s));
    TCG_HIP(hipStreamSynchronize(s));
    if (h_flag) return TCG_ECSR;

    hipLaunchKernelGGL(parent_kernel, dim3(blocks_for((int64_t)n * kGroup, kThreads)), dim3(kThreads), 0, s, n, d_row_ptr,
                       d_col_idx, seed, parent, long_rows, counters + 1);
    hipLaunchKernelGGL(parent_long_kernel, dim3((unsigned)max_long), dim3(kThreads), 0, s, d_row_ptr, d_col_idx, seed,
                       parent, long_rows, counters + 1);
    hipLaunchKernelGGL(root_kernel, dim3(blocks_for(n)), dim3(256), 0, s, n, parent, label_a);
    TCG_TRY(launch_status("parent/root kernels"));
    int32_t *label = label_a, *other = label_b;
    for (int32_t r = 0; r < refine; ++r) {
        hipLaunchKernelGGL(refine_kernel, dim3(blocks_for(n, kThreads / kGroup)), dim3(kThreads), 0, s, n, d_row_ptr,
                           d_col_idx, label, other);
        std::swap(label, other);
    }
    TCG_TRY(launch_status("refine_kernel"));
    // nodes by (label, parent, id): stable sort by parent, then stable sort by label
    const int bits = bits_for(n);
    TCG_TRY(radix_sort_pairs(parent, nullptr, n, nullptr, bits, keys, order1, sort_scratch, s));
    hipLaunchKernelGGL(gather_i32_kernel, dim3(blocks_for(n)), dim3(256), 0, s, (int64_t)n, order1, label, keys2);
    TCG_TRY(radix_sort_pairs(keys2, order1, n, nullptr, bits, keys, d_perm, sort_scratch, s));
    TCG_HIP(hipStreamSynchronize(s));        // the scratch goes back to the pool on return
    return TCG_OK;
}

int csr_permute_impl(int32_t n, int64_t nnz, const int32_t *d_row_ptr, const int32_t *d_col_idx,
                     const int32_t *d_perm, int32_t *d_out_row_ptr, int32_t *d_out_col_idx, int32_t *d_edge_perm,
                     hipStream_t s)
{
    if (n == 0) {
        hipLaunchKernelGGL(fill_kernel, dim3(1), dim3(64), 0, s, d_out_row_ptr, (int64_t)1, 0);
        return launch_status("fill_kernel");
    }
    const size_t arr = ((size_t)n * 4 + 255) & ~(size_t)255;
    const size_t scan_bytes = (size_t)scan_workspace_elems(n) * 4;
    PoolBuf buf;
    buf.s = s;
    TCG_TRY(pool_alloc(&buf.p, 2 * arr + 256 + scan_bytes));
    char *base = static_cast<char *>(buf.p);
    int32_t *inv = reinterpret_cast<int32_t *>(base);
    int32_t *deg = reinterpret_cast<int32_t *>(base + arr);
    int32_t *flag = reinterpret_cast<int32_t *>(base + 2 * arr);
    int32_t *scan_work = reinterpret_cast<int32_t *>(base + 2 * arr + 256);

    hipLaunchKernelGGL(fill_kernel, dim3(1), dim3(64), 0, s, flag, (int64_t)1, 0);
    hipLaunchKernelGGL(check_square_kernel, dim3((unsigned)std::min<int64_t>(ceil_div(std::max<int64_t>(nnz, n + 1), 256), 8192)),
                       dim3(256), 0, s, n, nnz, d_row_ptr, d_col_idx, flag);
    TCG_TRY(launch_status("check_square_kernel"));
    int h_flag = 0;
    TCG_HIP(hipMemcpyAsync(&h_flag, flag, sizeof(int), hipMemcpyDeviceToHost, s));
    TCG_HIP(hipStreamSynchronize(s));
    if (h_flag) return TCG_ECSR;

    hipLaunchKernelGGL(fill_kernel, dim3(blocks_for(n)), dim3(256), 0, s, inv, (int64_t)n, -1);
    hipLaunchKernelGGL(invert_perm_kernel, dim3(blocks_for(n)), dim3(256), 0, s, n, d_perm, d_row_ptr, inv, deg, flag);
    TCG_TRY(launch_status("invert_perm_kernel"));
    TCG_HIP(hipMemcpyAsync(&h_flag, flag, sizeof(int), hipMemcpyDeviceToHost, s));
    TCG_HIP(hipStreamSynchronize(s));
    if (h_flag) return TCG_EINVAL;           // not a permutation of the nodes

    TCG_TRY(exclusive_scan_i32(deg, d_out_row_ptr, n, scan_work, s));
    hipLaunchKernelGGL(set_last_kernel, dim3(1), dim3(1), 0, s, d_out_row_ptr, (int64_t)n, (int32_t)nnz);
    if (nnz > 0)
        hipLaunchKernelGGL(permute_entries_kernel, dim3(blocks_for(nnz)), dim3(256), 0, s, n, nnz, d_row_ptr, d_col_idx,
                           d_perm, inv, d_out_row_ptr, d_out_col_idx, d_edge_perm);
    TCG_TRY(launch_status("permute_entries_kernel"));
    TCG_HIP(hipStreamSynchronize(s));        // the scratch goes back to the pool on return
    return TCG_OK;
}

}  // namespace tcg
