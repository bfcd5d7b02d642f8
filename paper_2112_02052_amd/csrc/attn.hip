// Fused attention-style aggregation: Y[i] = sum_e softmax_i(<x_i, x_j>)_e * x_j, i.e. the chain
// SDDMM (Equation 2) -> row softmax -> SpMM (Equation 1) of the paper's AGNN workload in one pass.
// With per-node factors r and a scale beta the score of an edge becomes beta * r_i * r_j * <x_i, x_j>: with
// r = 1 / |x| that is the cosine attention of the AGNN layer, computed while x_j itself (not its normalised
// copy) is gathered once for score and aggregation alike.
//
// Run as three library calls the chain gathers every neighbour row twice (once for the score, once
// for the aggregation) and moves the scores through HBM three times.  Here a group of G lanes walks a
// row segment once: the 16-byte slices of a gathered row x_j sit in registers, the score is reduced
// across the group with wavefront shuffles, and the row is added to the accumulator under an online
// softmax (running maximum m and denominator l; the accumulator is rescaled whenever m grows), so the
// scores never leave the registers.  Rows split over several segments write (accumulator, m, l) per
// segment and a second kernel merges them in segment order: m = max m_s, l = sum l_s e^(m_s - m),
// y = sum y_s e^(m_s - m), Y = y / l.  Deterministic; rows without entries give 0.
#include "common.h"
#include "devutil.h"

namespace tcg {

namespace {

constexpr int kBlock = 256;

template <int DT, int G, int NCH, int UNROLL, bool HAS_R>
__global__ __launch_bounds__(kBlock) void attn_fused_kernel(
    const int32_t *__restrict__ lane_tab, const int32_t *__restrict__ seg_row, const int32_t *__restrict__ seg_ebeg,
    const int32_t *__restrict__ seg_dst, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
    const char *__restrict__ X, int64_t ldx_bytes, int32_t n_chunks, int32_t D, const float *__restrict__ rnorm,
    float beta, float *__restrict__ scores, void *__restrict__ Y, int y_dt, int64_t ldy, float *__restrict__ partial,
    float *__restrict__ partial_ml)
{
    constexpr int VEC = Elem<DT>::VEC;
    const int lane = threadIdx.x % G;
    const int64_t seg = plan_segment(lane_tab, kBlock / G, threadIdx.x / G);
    if (seg < 0) return;
    const int32_t row = seg_row[seg];
    const int32_t eb = seg_ebeg[seg];
    const int32_t dst = seg_dst[seg];
    const int32_t ee = segment_end(eb, dst, row, row_ptr);

    float xi[NCH][VEC], acc[NCH][VEC];
    {
        const char *xr = X + (int64_t)row * ldx_bytes;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int chunk = lane + c * G;
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (chunk < n_chunks && eb < ee)           // a row without entries only has its zeros written
                raw = *reinterpret_cast<const uint4 *>(xr + (int64_t)chunk * 16);
            unpack16<DT>(raw, xi[c]);
#pragma unroll
            for (int k = 0; k < VEC; ++k) acc[c][k] = 0.f;
        }
    }
    float m_run = -INFINITY, l_run = 0.f;
    const float r_i = HAS_R ? rnorm[row] : 1.f;

    if (eb < ee) {
        const int32_t last = ee - 1;
        const uint32_t ldx32 = (uint32_t)ldx_bytes;
        // ids: loaded once per lane group (lane l takes entries l, l + G, ...) and handed round with shuffles
        constexpr int PER = (UNROLL + G - 1) / G;
        auto request = [&](int32_t e0, int32_t (&mc)[PER]) {
#pragma unroll
            for (int k = 0; k < PER; ++k) mc[k] = col_idx[min(e0 + lane + k * G, last)];
        };
        auto hand_round = [&](const int32_t (&mc)[PER], int32_t (&c)[UNROLL]) {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) c[u] = __shfl(mc[u / G], u % G, G);
        };
        int32_t cn[UNROLL];
        {
            int32_t mc[PER];
            request(eb, mc);
            hand_round(mc, cn);
        }
        for (int32_t e = eb; e < ee; e += UNROLL) {
            int32_t mc_next[PER];
            request(e + UNROLL, mc_next);
            float v[UNROLL][NCH][VEC];
            float p[UNROLL], rj[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const char *xr = X + (uint64_t)(uint32_t)cn[u] * ldx32;
                rj[u] = HAS_R ? rnorm[cn[u]] : 1.f;         // the same address in every lane of the group
                float a = 0.f;
#pragma unroll
                for (int c = 0; c < NCH; ++c) {
                    const int chunk = lane + c * G;
                    uint4 raw = make_uint4(0, 0, 0, 0);
                    if (e + u < ee && chunk < n_chunks) raw = *reinterpret_cast<const uint4 *>(xr + (uint32_t)chunk * 16u);
                    unpack16<DT>(raw, v[u][c]);
#pragma unroll
                    for (int k = 0; k < VEC; ++k) a = fmaf(xi[c][k], v[u][c][k], a);
                }
                p[u] = a;
            }
            hand_round(mc_next, cn);          // after the row loads have gone out

            // Scores of the UNROLL edges, known to every lane of the group: the stored score is
            // r_i * r_j * <x_i, x_j>, the softmax runs over beta times that.
            float s[UNROLL];
            const float r = group_reduce<G, UNROLL>(p, lane);
            if constexpr (G >= UNROLL) {
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) s[u] = __shfl(r, u, G);
            } else {
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) s[u] = p[u];
            }
            if constexpr (HAS_R) {
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) s[u] *= r_i * rj[u];
            }
            if (scores != nullptr) {
                if constexpr (G >= UNROLL) {        // lane u stores the score of edge u: one coalesced store
                    float mine = s[0];
#pragma unroll
                    for (int u = 1; u < UNROLL; ++u) mine = lane == u ? s[u] : mine;
                    if (lane < UNROLL && e + lane < ee) scores[e + lane] = mine;
                } else if (lane == 0) {
#pragma unroll
                    for (int u = 0; u < UNROLL; ++u)
                        if (e + u < ee) scores[e + u] = s[u];
                }
            }
            if constexpr (HAS_R) {
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) s[u] *= beta;
            }
            // Online softmax update (edge e itself is always valid, so the new maximum is finite).
            float m_new = m_run;
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
                if (e + u < ee) m_new = fmaxf(m_new, s[u]);
            const float scale = expf(m_run - m_new);      // 0 for the first chunk (m_run = -inf)
            l_run *= scale;
#pragma unroll
            for (int c = 0; c < NCH; ++c)
#pragma unroll
                for (int k = 0; k < VEC; ++k) acc[c][k] *= scale;
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const float wgt = (e + u < ee) ? expf(s[u] - m_new) : 0.f;
                l_run += wgt;
#pragma unroll
                for (int c = 0; c < NCH; ++c)
#pragma unroll
                    for (int k = 0; k < VEC; ++k) acc[c][k] = fmaf(wgt, v[u][c][k], acc[c][k]);
            }
            m_run = m_new;
        }
    }

    const float inv = (dst < 0 && l_run > 0.f) ? 1.f / l_run : (dst < 0 ? 0.f : 1.f);
    if (dst >= 0 && lane == 0) {
        partial_ml[2 * (int64_t)segment_slot(dst)] = m_run;
        partial_ml[2 * (int64_t)segment_slot(dst) + 1] = l_run;
    }
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int chunk = lane + c * G;
        if (chunk >= n_chunks) continue;
        const int64_t d0 = (int64_t)chunk * VEC;
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            const float val = acc[c][k] * inv;
            if (dst >= 0) partial[(int64_t)segment_slot(dst) * D + d0 + k] = val;
            else store_elem(Y, (int64_t)row * ldy + d0 + k, y_dt, val);
        }
    }
}

// Merges the per-segment (accumulator, maximum, denominator) of every split row: one workgroup per row.  The
// row's maximum and denominator come from a workgroup-wide reduction over its segments; for the accumulators a
// thread takes four columns, so D / 4 threads cover a partial row and the 256 / (D / 4) thread groups each add
// every such-and-such segment, their sums meeting in LDS in group order.  The order of all additions is fixed
// by the sizes alone, so results repeat from run to run.  (One thread per column walking all segments one after
// the other made this kernel as long as the fused kernel itself: a hub row has hundreds of segments.)
__device__ __forceinline__ float block_reduce(float v, float *s_red, bool is_max)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const float t = __shfl_xor(v, off, kWave);
        v = is_max ? fmaxf(v, t) : v + t;
    }
    __syncthreads();                         // s_red may still be read from the previous reduction
    if (lane == 0) s_red[wave] = v;
    __syncthreads();
    float r = s_red[0];
#pragma unroll
    for (int i = 1; i < kBlock / kWave; ++i) r = is_max ? fmaxf(r, s_red[i]) : r + s_red[i];
    return r;
}

__global__ __launch_bounds__(kBlock) void attn_merge_long_kernel(
    const int32_t *__restrict__ long_row, const int32_t *__restrict__ long_slot_ptr, const float *__restrict__ partial,
    const float *__restrict__ partial_ml, int32_t D, void *__restrict__ Y, int y_dt, int64_t ldy)
{
    __shared__ float s_red[kBlock / kWave];
    __shared__ float4 s_part[kBlock];
    const int64_t li = blockIdx.x;
    const int32_t row = long_row[li];
    const int32_t s0 = long_slot_ptr[li], s1 = long_slot_ptr[li + 1];
    float m = -INFINITY;
    for (int32_t sgi = s0 + threadIdx.x; sgi < s1; sgi += kBlock) m = fmaxf(m, partial_ml[2 * (int64_t)sgi]);
    m = block_reduce(m, s_red, true);
    float l = 0.f;
    for (int32_t sgi = s0 + threadIdx.x; sgi < s1; sgi += kBlock)
        l += partial_ml[2 * (int64_t)sgi + 1] * expf(partial_ml[2 * (int64_t)sgi] - m);
    l = block_reduce(l, s_red, false);
    const float inv = l > 0.f ? 1.f / l : 0.f;
    const int32_t c4 = D / 4;
    if (D % 4 == 0 && c4 <= kBlock) {
        const int32_t nsg = kBlock / c4;
        const int32_t c = threadIdx.x % c4, sg = threadIdx.x / c4;
        float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
        if (sg < nsg)
            for (int32_t sgi = s0 + sg; sgi < s1; sgi += nsg) {
                const float w = expf(partial_ml[2 * (int64_t)sgi] - m);
                const float4 v = *reinterpret_cast<const float4 *>(partial + (int64_t)sgi * D + 4 * c);
                a.x = fmaf(v.x, w, a.x);
                a.y = fmaf(v.y, w, a.y);
                a.z = fmaf(v.z, w, a.z);
                a.w = fmaf(v.w, w, a.w);
            }
        s_part[threadIdx.x] = a;
        __syncthreads();
        if (sg == 0) {
            float4 t = s_part[c];
            for (int32_t g = 1; g < nsg; ++g) {
                const float4 v = s_part[g * c4 + c];
                t.x += v.x;
                t.y += v.y;
                t.z += v.z;
                t.w += v.w;
            }
            const int64_t o = (int64_t)row * ldy + 4 * c;
            store_elem(Y, o, y_dt, t.x * inv);
            store_elem(Y, o + 1, y_dt, t.y * inv);
            store_elem(Y, o + 2, y_dt, t.z * inv);
            store_elem(Y, o + 3, y_dt, t.w * inv);
        }
        return;
    }
    for (int32_t d = threadIdx.x; d < D; d += kBlock) {
        float y = 0.f;
        for (int32_t sgi = s0; sgi < s1; ++sgi)
            y = fmaf(partial[(int64_t)sgi * D + d], expf(partial_ml[2 * (int64_t)sgi] - m), y);
        store_elem(Y, (int64_t)row * ldy + d, y_dt, y * inv);
    }
}

struct Args {
    tcg_meta *m;
    const void *X;
    int64_t ldx;
    int32_t D;
    const float *rnorm;
    float beta;
    float *scores;
    void *Y;
    int y_dt;
    int64_t ldy;
    float *partial_ml;
    hipStream_t s;
};

template <int DT, int G, int NCH>
void launch(const Args &a, int32_t n_chunks)
{
    constexpr int UNROLL = NCH == 1 ? 8 : (NCH == 2 ? 4 : 2);
    const tcg_meta *m = a.m;
    const unsigned grid = (unsigned)plan_grid(m->h_lane_tab, kBlock / G);
    if (a.rnorm)
        hipLaunchKernelGGL((attn_fused_kernel<DT, G, NCH, UNROLL, true>), dim3(grid), dim3(kBlock), 0, a.s, m->d_lane_tab,
                           m->d_seg_row, m->d_seg_ebeg, m->d_seg_dst, m->d_row_ptr, m->d_col_idx,
                           static_cast<const char *>(a.X), a.ldx * Elem<DT>::BYTES, n_chunks, a.D, a.rnorm, a.beta,
                           a.scores, a.Y, a.y_dt, a.ldy, m->d_partial, a.partial_ml);
    else
        hipLaunchKernelGGL((attn_fused_kernel<DT, G, NCH, UNROLL, false>), dim3(grid), dim3(kBlock), 0, a.s, m->d_lane_tab,
                           m->d_seg_row, m->d_seg_ebeg, m->d_seg_dst, m->d_row_ptr, m->d_col_idx,
                           static_cast<const char *>(a.X), a.ldx * Elem<DT>::BYTES, n_chunks, a.D, a.rnorm, a.beta,
                           a.scores, a.Y, a.y_dt, a.ldy, m->d_partial, a.partial_ml);
}

template <int DT>
bool dispatch(const Args &a, int32_t n_chunks)
{
    if (n_chunks <= 4) launch<DT, 4, 1>(a, n_chunks);
    else if (n_chunks <= 8) launch<DT, 8, 1>(a, n_chunks);
    else if (n_chunks <= 16) launch<DT, 16, 1>(a, n_chunks);
    else if (n_chunks <= 32) launch<DT, 32, 1>(a, n_chunks);
    else if (n_chunks <= 64) launch<DT, 64, 1>(a, n_chunks);
    else if (n_chunks <= 128) launch<DT, 64, 2>(a, n_chunks);
    else return false;
    return true;
}

}  // namespace

// out[i] = 1 / max(|x_i|, eps): 16 lanes per row.
__global__ __launch_bounds__(256) void row_rnorm_kernel(int64_t n, const void *__restrict__ X, int x_dt, int32_t D,
                                                        int64_t ldx, float eps, float *__restrict__ out)
{
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) / 16;
    const int gl = threadIdx.x % 16;
    float a = 0.f;
    if (i < n)
        for (int32_t d = gl; d < D; d += 16) {
            const float v = load_elem(X, i * ldx + d, x_dt);
            a = fmaf(v, v, a);
        }
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) a += __shfl_xor(a, off, kWave);
    if (i < n && gl == 0) out[i] = 1.f / fmaxf(sqrtf(a), eps);
}

int row_rnorm_impl(int64_t n, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, float eps, float *d_out,
                   hipStream_t s)
{
    if (n == 0) return TCG_OK;
    hipLaunchKernelGGL(row_rnorm_kernel, dim3((unsigned)ceil_div(n * 16, 256)), dim3(256), 0, s, n, d_X, (int)x_dt, D, ldx,
                       eps, d_out);
    return launch_status("row_rnorm_kernel");
}

// dX[i] += scale * r_i * (G[i] - xn_i <G[i], xn_i>), xn_i = r_i x_i: 16 lanes per row, the row's dot product first.
__global__ __launch_bounds__(256) void row_unit_grad_kernel(int64_t n, const void *__restrict__ X, int x_dt, int32_t D,
                                                            int64_t ldx, const float *__restrict__ rnorm, float scale,
                                                            const float *__restrict__ G, int64_t ldg,
                                                            float *__restrict__ dX, int64_t ldd)
{
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) / 16;
    const int gl = threadIdx.x % 16;
    float dot = 0.f;
    if (i < n)
        for (int32_t d = gl; d < D; d += 16) dot = fmaf(G[i * ldg + d], load_elem(X, i * ldx + d, x_dt), dot);
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) dot += __shfl_xor(dot, off, kWave);
    if (i >= n) return;
    const float r = rnorm[i];
    const float back = r * r * dot;                      // <G, xn> r: the factor of x in xn <G, xn>
    for (int32_t d = gl; d < D; d += 16)
        dX[i * ldd + d] += scale * r * (G[i * ldg + d] - back * load_elem(X, i * ldx + d, x_dt));
}

int row_unit_grad_impl(int64_t n, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, const float *d_rnorm,
                       float scale, const float *d_G, int64_t ldg, float *d_dX, int64_t ldd, hipStream_t s)
{
    if (n == 0) return TCG_OK;
    hipLaunchKernelGGL(row_unit_grad_kernel, dim3((unsigned)ceil_div(n * 16, 256)), dim3(256), 0, s, n, d_X, (int)x_dt, D,
                       ldx, d_rnorm, scale, d_G, ldg, d_dX, ldd);
    return launch_status("row_unit_grad_kernel");
}

int attention_impl(tcg_meta *m, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, const float *d_rnorm, float beta,
                   float *d_scores, void *d_Y, tcg_dtype y_dt, int64_t ldy, hipStream_t s)
{
    if (m->n_rows == 0) return TCG_OK;
    const int es = dtype_size(x_dt);
    const bool vec_ok = ((int64_t)D * es) % 16 == 0 && (ldx * es) % 16 == 0 && ldx * es < (1ll << 32) &&
                        (reinterpret_cast<uintptr_t>(d_X) & 15) == 0 && (int64_t)D * es / 16 <= 128;
    if (!vec_ok) return TCG_EINVAL;

    // Scratch: fp32 accumulators of split rows (shared with tcg_spmm) and their (max, denominator).
    TCG_TRY(reserve_partial(m, D, s));

    Args a{m, d_X, ldx, D, d_rnorm, beta, d_scores, d_Y, (int)y_dt, ldy, m->d_partial_ml, s};
    const int32_t n_chunks = (int32_t)((int64_t)D * es / 16);
    bool ok;
    if (x_dt == TCG_F32) ok = dispatch<TCG_F32>(a, n_chunks);
    else if (x_dt == TCG_BF16) ok = dispatch<TCG_BF16>(a, n_chunks);
    else ok = dispatch<TCG_F16>(a, n_chunks);
    if (!ok) return TCG_EINVAL;
    TCG_TRY(launch_status("attn_fused_kernel"));
    if (m->n_long > 0) {
        hipLaunchKernelGGL(attn_merge_long_kernel, dim3((unsigned)m->n_long), dim3(kBlock), 0, s, m->d_long_row,
                           m->d_long_slot_ptr, m->d_partial, m->d_partial_ml, D, d_Y, (int)y_dt, ldy);
        TCG_TRY(launch_status("attn_merge_long_kernel"));
    }
    return TCG_OK;
}

}  // namespace tcg
