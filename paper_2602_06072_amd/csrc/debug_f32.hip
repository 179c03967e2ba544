// fp32 debug path: plain FMA attention, one wave per (query row, head), and a
// plain gather for the fp32 buffer layout.  Straightforward mapping, no MFMA;
// it exists to check the plan, the tables and the layouts at 1e-4 accuracy.
#include "common.hip.h"
#include "kernels.h"

namespace pk {
namespace {

constexpr int kChunk = 1024;       // keys scored per pass
constexpr int kMaxAcc = 4;         // d <= 64 * kMaxAcc

struct RowState {
    float m;                       // running max of scaled scores
    float l;                       // running sum of exp(score - m)
    float acc[kMaxAcc];            // output columns lane, lane+64, ...
};

// One query row against `ntok` keys starting at k/v (token stride `tstride`
// floats).  q_s: the query in LDS; s_s: kChunk floats of LDS scratch.
__device__ void attend_segment(RowState& st, const float* q_s, float* s_s,
                               const float* __restrict__ k, const float* __restrict__ v,
                               int64_t ntok, int64_t tstride, int d, float scale) {
    const int lane = threadIdx.x;
    for (int64_t c0 = 0; c0 < ntok; c0 += kChunk) {
        const int cn = static_cast<int>(ntok - c0 < kChunk ? ntok - c0 : kChunk);
        float cmax = -INFINITY;
        for (int j = lane; j < cn; j += 64) {
            const float* kj = k + (c0 + j) * tstride;
            float s = 0.f;
            for (int c = 0; c < d; ++c) s = fmaf(q_s[c], kj[c], s);
            s *= scale;
            s_s[j] = s;
            cmax = fmaxf(cmax, s);
        }
        cmax = wave_max(cmax);
        const float m_new = fmaxf(st.m, cmax);
        const float alpha = (st.m == -INFINITY) ? 0.f : expf(st.m - m_new);
        __syncthreads();
        float lsum = 0.f;
        for (int j = lane; j < cn; j += 64) {
            const float p = expf(s_s[j] - m_new);
            s_s[j] = p;
            lsum += p;
        }
        lsum = wave_sum(lsum);
        st.l = st.l * alpha + lsum;
        st.m = m_new;
        __syncthreads();
#pragma unroll
        for (int a = 0; a < kMaxAcc; ++a) {
            const int col = lane + 64 * a;
            if (col < d) {
                float acc = st.acc[a] * alpha;
                for (int j = 0; j < cn; ++j) acc = fmaf(s_s[j], v[(c0 + j) * tstride + col], acc);
                st.acc[a] = acc;
            }
        }
        __syncthreads();
    }
}

__device__ void store_row(const RowState& st, void* out, int64_t row_elem0, int d, int out_f32) {
    const int lane = threadIdx.x;
    const float inv = st.l > 0.f ? 1.f / st.l : 0.f;
#pragma unroll
    for (int a = 0; a < kMaxAcc; ++a) {
        const int col = lane + 64 * a;
        if (col < d) {
            const float o = st.acc[a] * inv;
            if (out_f32) static_cast<float*>(out)[row_elem0 + col] = o;
            else static_cast<uint16_t*>(out)[row_elem0 + col] = float_to_bf16_bits(o);
        }
    }
}

__global__ __launch_bounds__(64) void prefill_f32_kernel(PrefillArgs a) {
    __shared__ float q_s[64 * kMaxAcc];
    __shared__ float s_s[kChunk];
    const int64_t row = blockIdx.x;
    const int h = blockIdx.y;
    int lo = 0, hi = a.n;                                   // request owning this row
    while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (a.q_start[mid] <= row) lo = mid; else hi = mid; }
    const int i = lo;
    const int64_t t = row - a.q_start[i];
    const int64_t lq = a.q_start[i + 1] - a.q_start[i];
    const int64_t lkv = a.kv_start[i + 1] - a.kv_start[i];
    const int g = h / (a.Hq / a.Hkv);
    const float* q = static_cast<const float*>(a.q) + (row * a.Hq + h) * a.d;
    for (int c = threadIdx.x; c < a.d; c += 64) q_s[c] = q[c];
    __syncthreads();
    RowState st; st.m = -INFINITY; st.l = 0.f;
#pragma unroll
    for (int x = 0; x < kMaxAcc; ++x) st.acc[x] = 0.f;
    const int64_t tstride = static_cast<int64_t>(a.Hkv) * a.d;
    const int64_t base = (static_cast<int64_t>(a.kv_start[i]) * a.Hkv + g) * a.d;
    attend_segment(st, q_s, s_s, static_cast<const float*>(a.k) + base,
                   static_cast<const float*>(a.v) + base, (lkv - lq) + t + 1, tstride, a.d, a.scale);
    store_row(st, a.out, (row * a.Hq + h) * a.d, a.d, a.out_f32);
}

__global__ __launch_bounds__(64) void decode_f32_kernel(DecodeArgs a) {
    __shared__ float q_s[64 * kMaxAcc];
    __shared__ float s_s[kChunk];
    const int i = blockIdx.x, h = blockIdx.y;
    const int g = h / (a.Hq / a.Hkv);
    const float* q = static_cast<const float*>(a.q) + (static_cast<int64_t>(i) * a.Hq + h) * a.d;
    for (int c = threadIdx.x; c < a.d; c += 64) q_s[c] = q[c];
    __syncthreads();
    RowState st; st.m = -INFINITY; st.l = 0.f;
#pragma unroll
    for (int x = 0; x < kMaxAcc; ++x) st.acc[x] = 0.f;
    const float* kb = static_cast<const float*>(a.kv_buf);
    const float* vb = kb + static_cast<int64_t>(a.Hkv) * a.buf_tokens * a.d;
    // the request's shared segments, outermost first, then its own suffix (Sec. 3.2, Eq. 5)
    for (int c = a.chain_start[i]; c < a.chain_start[i + 1]; ++c) {
        const int64_t off = (static_cast<int64_t>(g) * a.buf_tokens + a.chain[2 * c]) * a.d;
        attend_segment(st, q_s, s_s, kb + off, vb + off, a.chain[2 * c + 1], a.d, a.d, a.scale);
    }
    const int32_t* seg = a.req_seg + 4 * i;                 // prefix_off, L_P, suffix_off, L_Q (absolute)
    const int64_t off = (static_cast<int64_t>(g) * a.buf_tokens + seg[2]) * a.d;
    attend_segment(st, q_s, s_s, kb + off, vb + off, seg[3] + a.grown, a.d, a.d, a.scale);
    store_row(st, a.out, (static_cast<int64_t>(i) * a.Hq + h) * a.d, a.d, a.out_f32);
}

// fp32 buffer layout: K [Hkv][buf_tokens][d], then V.  One thread per element.
__global__ __launch_bounds__(256) void reorg_f32_kernel(ReorgArgs a) {
    const int64_t tok = blockIdx.x;                          // buffer token
    const int blk = static_cast<int>(tok / 32);
    int s = a.blk_first[blk];
    while (s < a.n_seg && static_cast<int64_t>(a.seg[4 * s]) + a.seg[4 * s + 1] <= tok) ++s;
    if (s >= a.n_seg || a.seg[4 * s] > tok) return;          // hole: leave untouched
    const int req = a.seg[4 * s + 2];
    const int64_t pos = a.seg[4 * s + 3] + (tok - a.seg[4 * s]);
    int64_t page = a.block_table[static_cast<int64_t>(req) * a.max_blocks + pos / a.page_size];
    page = page < 0 ? 0 : (page >= a.num_blocks ? a.num_blocks - 1 : page);
    const int64_t src = (page * a.page_size + pos % a.page_size) * a.Hkv * a.d;
    const float* kp = static_cast<const float*>(a.k_pages) + src;
    const float* vp = static_cast<const float*>(a.v_pages) + src;
    float* kb = static_cast<float*>(a.kv_buf);
    float* vb = kb + static_cast<int64_t>(a.Hkv) * a.buf_tokens * a.d;
    for (int e = threadIdx.x; e < a.Hkv * a.d; e += blockDim.x) {
        const int h = e / a.d, c = e % a.d;
        const int64_t dst = (static_cast<int64_t>(h) * a.buf_tokens + tok) * a.d + c;
        kb[dst] = kp[e];
        vb[dst] = vp[e];
    }
}

// the token of decode step `step` into its request's headroom (fp32 layout)
__global__ __launch_bounds__(256) void append_f32_kernel(AppendArgs a) {
    const int i = blockIdx.x, h = blockIdx.y;
    const int32_t* seg = a.req_seg + 4 * i;
    const int64_t tok = static_cast<int64_t>(seg[2]) + seg[3] + a.step;
    float* kb = static_cast<float*>(a.kv_buf);
    float* vb = kb + static_cast<int64_t>(a.Hkv) * a.buf_tokens * a.d;
    const int64_t src = (static_cast<int64_t>(i) * a.Hkv + h) * a.d;
    const int64_t dst = (static_cast<int64_t>(h) * a.buf_tokens + tok) * a.d;
    for (int c = threadIdx.x; c < a.d; c += blockDim.x) {
        kb[dst + c] = static_cast<const float*>(a.k_new)[src + c];
        vb[dst + c] = static_cast<const float*>(a.v_new)[src + c];
    }
}

}  // namespace

int launch_append_f32(const AppendArgs& a, void* stream) {
    if (a.n == 0) return 0;
    hipLaunchKernelGGL(append_f32_kernel, dim3(static_cast<unsigned>(a.n), static_cast<unsigned>(a.Hkv)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), a);
    return static_cast<int>(hipGetLastError());
}

int launch_prefill_f32(const PrefillArgs& a, void* stream) {
    if (a.total_q_rows == 0) return 0;
    dim3 grid(static_cast<unsigned>(a.total_q_rows), static_cast<unsigned>(a.Hq));
    hipLaunchKernelGGL(prefill_f32_kernel, grid, dim3(64), 0, static_cast<hipStream_t>(stream), a);
    return static_cast<int>(hipGetLastError());
}

int launch_decode_f32(const DecodeArgs& a, void* stream) {
    if (a.n == 0) return 0;
    dim3 grid(static_cast<unsigned>(a.n), static_cast<unsigned>(a.Hq));
    hipLaunchKernelGGL(decode_f32_kernel, grid, dim3(64), 0, static_cast<hipStream_t>(stream), a);
    return static_cast<int>(hipGetLastError());
}

int launch_reorg_f32(const ReorgArgs& a, void* stream) {
    if (a.buf_tokens == 0) return 0;
    hipLaunchKernelGGL(reorg_f32_kernel, dim3(static_cast<unsigned>(a.buf_tokens)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), a);
    return static_cast<int>(hipGetLastError());
}

}  // namespace pk
