// Stable least-significant-digit radix sort of (key, value) pairs with 8-bit digits, used by the CSR
// transpose (entries by column), the row clustering and the ordering of the gather plan.  It is the
// library's own sort so that results are unique and repeat bit for bit.
//
// One pass = three steps: per-tile digit counts, an exclusive scan of the counts in digit-major order, and a
// stable scatter.  A tile is THREADS * KPT consecutive keys handled by one workgroup; a wavefront owns a
// contiguous piece of it and walks it in rounds of 64 keys.  In the scatter the rank of a key among the
// tile's keys with the same digit is (keys of earlier wavefronts) + (keys of earlier rounds of this
// wavefront) + (lower lanes of this round), the last two from wavefront ballots over the digit's bits.
// The tile is then put in digit order in LDS first, so that neighbouring threads write neighbouring
// output positions: with 256 digits a tile's run per digit is short, and scattering straight from
// registers would write 4 bytes at a time.
#include "common.h"

namespace tcg {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kDigitBits = 8;
constexpr int kDigits = 1 << kDigitBits;

__device__ __forceinline__ int64_t effective_n(int64_t n_max, const int32_t *d_n)
{
    if (!d_n) return n_max;
    const int64_t v = *d_n;
    return v < n_max ? (v < 0 ? 0 : v) : n_max;
}

// Step 1: block_cnt[digit * n_blocks + block].
template <int KPT>
__global__ __launch_bounds__(kThreads) void radix_count_kernel(const int32_t *__restrict__ keys, int64_t n_max,
                                                               const int32_t *__restrict__ d_n, int shift,
                                                               int32_t *__restrict__ block_cnt, int64_t n_blocks)
{
    __shared__ int s_cnt[kDigits];
    s_cnt[threadIdx.x] = 0;
    __syncthreads();
    const int64_t n = effective_n(n_max, d_n);
    const int64_t base = (int64_t)blockIdx.x * (kThreads * KPT);
    int32_t k[KPT];
#pragma unroll
    for (int r = 0; r < KPT; ++r) {
        const int64_t i = base + r * kThreads + threadIdx.x;
        k[r] = i < n ? keys[i] : -1;
    }
#pragma unroll
    for (int r = 0; r < KPT; ++r)
        if (k[r] >= 0) atomicAdd(&s_cnt[(k[r] >> shift) & (kDigits - 1)], 1);
    __syncthreads();
    block_cnt[(int64_t)threadIdx.x * n_blocks + blockIdx.x] = s_cnt[threadIdx.x];
}

// Step 3.  block_off = exclusive scan of block_cnt.  vals_in == nullptr stands for the identity.
template <int KPT>
__global__ __launch_bounds__(kThreads) void radix_scatter_kernel(
    const int32_t *__restrict__ keys_in, const int32_t *__restrict__ vals_in, int64_t n_max,
    const int32_t *__restrict__ d_n, int shift, const int32_t *__restrict__ block_off, int64_t n_blocks,
    int32_t *__restrict__ keys_out, int32_t *__restrict__ vals_out)
{
    constexpr int TILE = kThreads * KPT;
    __shared__ int s_cnt[kWaves][kDigits];       // per wavefront: running count, then offset of the wavefront
    __shared__ int s_start[kDigits];             // first tile-local position of a digit
    __shared__ int32_t s_base[kDigits];          // first output position of the tile's keys with a digit
    __shared__ int s_tmp[kWaves + 1];
    __shared__ int32_t s_keys[TILE], s_vals[TILE];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int64_t n = effective_n(n_max, d_n);
    const int64_t tile_base = (int64_t)blockIdx.x * TILE;
    if (tile_base >= n) return;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) s_cnt[w][threadIdx.x] = 0;
    __syncthreads();

    int32_t key[KPT], val[KPT];
    int rank[KPT];
#pragma unroll
    for (int r = 0; r < KPT; ++r) {
        const int64_t i = tile_base + (int64_t)wave * (kWave * KPT) + r * kWave + lane;
        key[r] = i < n ? keys_in[i] : -1;
        val[r] = i < n ? (vals_in ? vals_in[i] : (int32_t)i) : 0;
    }
#pragma unroll
    for (int r = 0; r < KPT; ++r) {
        const bool valid = key[r] >= 0;
        const int d = (key[r] >> shift) & (kDigits - 1);
        unsigned long long same = __ballot(valid);
#pragma unroll
        for (int b = 0; b < kDigitBits; ++b) {
            const unsigned long long bal = __ballot((d >> b) & 1);
            same &= ((d >> b) & 1) ? bal : ~bal;
        }
        rank[r] = 0;
        if (valid) {
            const int before = s_cnt[wave][d];           // keys of this digit in this wavefront's earlier rounds
            rank[r] = before + __popcll(same & ((1ull << lane) - 1ull));
            if ((same & ((1ull << lane) - 1ull)) == 0) s_cnt[wave][d] = before + __popcll(same);
        }
        __builtin_amdgcn_wave_barrier();                 // the next round reads what this one wrote
    }
    __syncthreads();
    // thread d: offsets of the wavefronts inside digit d, the digit's place in the tile and in the output
    int tot = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const int c = s_cnt[w][threadIdx.x];
        s_cnt[w][threadIdx.x] = tot;
        tot += c;
    }
    // exclusive scan of the digit totals over the 256 threads
    int incl = tot;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int t = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += t;
    }
    if (lane == kWave - 1) s_tmp[wave] = incl;
    __syncthreads();
    int wave_off = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w)
        if (w < wave) wave_off += s_tmp[w];
    s_start[threadIdx.x] = wave_off + incl - tot;
    s_base[threadIdx.x] = block_off[(int64_t)threadIdx.x * n_blocks + blockIdx.x];
    __syncthreads();
#pragma unroll
    for (int r = 0; r < KPT; ++r) {
        if (key[r] < 0) continue;
        const int d = (key[r] >> shift) & (kDigits - 1);
        const int p = s_start[d] + s_cnt[wave][d] + rank[r];
        s_keys[p] = key[r];
        s_vals[p] = val[r];
    }
    __syncthreads();
    const int count = (int)(n - tile_base < TILE ? n - tile_base : TILE);
    for (int i = threadIdx.x; i < count; i += kThreads) {
        const int32_t k = s_keys[i];
        const int d = (k >> shift) & (kDigits - 1);
        const int64_t g = (int64_t)s_base[d] + (i - s_start[d]);
        keys_out[g] = k;
        vals_out[g] = s_vals[i];
    }
}

constexpr int kKeysSmall = 4, kKeysLarge = 16;       // keys per thread: tiles of 1024 / 4096 keys
constexpr int64_t kLargeFrom = 1 << 16;

inline int keys_per_thread(int64_t n_max) { return n_max >= kLargeFrom ? kKeysLarge : kKeysSmall; }

}  // namespace

size_t radix_sort_scratch_bytes(int64_t n_max)
{
    const int64_t n_blocks = ceil_div(std::max<int64_t>(n_max, 1), kThreads * keys_per_thread(n_max));
    const int64_t cnt_elems = (int64_t)kDigits * n_blocks + 1;
    if (cnt_elems >= (int64_t)INT32_MAX) return 0;
    const size_t arr = ((size_t)std::max<int64_t>(n_max, 1) * 4 + 255) & ~(size_t)255;
    const size_t cnt_bytes = ((size_t)cnt_elems * 4 + 255) & ~(size_t)255;
    return 2 * arr + cnt_bytes + (size_t)scan_workspace_elems(cnt_elems) * 4;
}

int radix_sort_pairs(const int32_t *d_keys_in, const int32_t *d_vals_in, int64_t n_max, const int32_t *d_n, int bits,
                     int32_t *d_keys_out, int32_t *d_vals_out, void *d_scratch, hipStream_t s)
{
    if (n_max == 0) return TCG_OK;
    const int passes = std::max(1, (bits + kDigitBits - 1) / kDigitBits);
    const int kpt = keys_per_thread(n_max);
    const int64_t n_blocks = ceil_div(n_max, kThreads * kpt);
    const int64_t cnt_elems = (int64_t)kDigits * n_blocks + 1;
    const size_t arr = ((size_t)n_max * 4 + 255) & ~(size_t)255;
    const size_t cnt_bytes = ((size_t)cnt_elems * 4 + 255) & ~(size_t)255;
    char *base = static_cast<char *>(d_scratch);
    int32_t *keys_b = reinterpret_cast<int32_t *>(base);
    int32_t *vals_b = reinterpret_cast<int32_t *>(base + arr);
    int32_t *block_cnt = reinterpret_cast<int32_t *>(base + 2 * arr);
    int32_t *scan_work = reinterpret_cast<int32_t *>(base + 2 * arr + cnt_bytes);

    const int32_t *kin = d_keys_in;
    const int32_t *vin = d_vals_in;
    for (int pass = 0; pass < passes; ++pass) {
        // Choose the outputs so that the last pass lands in the caller's arrays.
        const bool to_out = ((passes - 1 - pass) % 2) == 0;
        int32_t *kout = to_out ? d_keys_out : keys_b;
        int32_t *vout = to_out ? d_vals_out : vals_b;
        const int shift = kDigitBits * pass;
        if (kpt == kKeysLarge)
            hipLaunchKernelGGL(radix_count_kernel<kKeysLarge>, dim3((unsigned)n_blocks), dim3(kThreads), 0, s, kin, n_max,
                               d_n, shift, block_cnt, n_blocks);
        else
            hipLaunchKernelGGL(radix_count_kernel<kKeysSmall>, dim3((unsigned)n_blocks), dim3(kThreads), 0, s, kin, n_max,
                               d_n, shift, block_cnt, n_blocks);
        TCG_TRY(exclusive_scan_i32(block_cnt, block_cnt, cnt_elems - 1, scan_work, s));
        if (kpt == kKeysLarge)
            hipLaunchKernelGGL(radix_scatter_kernel<kKeysLarge>, dim3((unsigned)n_blocks), dim3(kThreads), 0, s, kin, vin,
                               n_max, d_n, shift, block_cnt, n_blocks, kout, vout);
        else
            hipLaunchKernelGGL(radix_scatter_kernel<kKeysSmall>, dim3((unsigned)n_blocks), dim3(kThreads), 0, s, kin, vin,
                               n_max, d_n, shift, block_cnt, n_blocks, kout, vout);
        TCG_TRY(launch_status("radix kernels"));
        kin = kout;
        vin = vout;
    }
    return TCG_OK;
}

}  // namespace tcg
