// Paged GQA decode attention over the shared pool (gfx950 / CDNA4).
//
// Defines out = softmax(q K^T / sqrt(D)) V per sequence and query head, with K and V
// read through the sequence's block-table row (paper: Background, "KV cache and
// PagedAttention"; the balloon driver leaves attention semantics untouched, Sec. 4.2
// R4/D4).  The path is bound by HBM reads of K and V, each byte exactly once.
//
// Mapping to the hardware
//   * one wavefront (64 lanes) per work item = (sequence, kv head, chunk of pages):
//     split-K over pages, merged afterwards with the online-softmax rule;
//   * K and V tiles are stored inside a block in the lane order of the MFMA operands,
//     so each 16-byte global load is fully coalesced (64 lanes x 16 B = 1 KiB
//     contiguous) and lands directly in operand registers — no LDS round trip, no
//     shuffles between load and matrix op;
//   * the g query heads that share a kv head are padded to the 16 columns of one
//     MFMA tile: S[token][head] = K . q^T is a 16x16x32 bf16 MFMA per 32 elements of
//     head_dim, and out^T[d][head] += V^T . P is a 16x16x16 bf16 MFMA per 16 elements
//     of head_dim, with P split into bf16 high and low parts (two MFMAs) so that the
//     probabilities keep 16 significant bits; accumulation is fp32 throughout;
//   * the softmax runs on the MFMA accumulator layout (lane = 4 tokens x 1 head):
//     in-lane max / sum plus two cross-lane steps per page.
//
// In-block layout (per kv head: K tile then V tile, T = 16 tokens):
//   bf16 K: 16-byte unit (c, t)      = K[t][8c .. 8c+7]                 at ((c*16)+t)*16
//   bf16 V: 16-byte unit (jp, G, dl) = V[4G..4G+3][32jp+dl] ,
//                                      V[4G..4G+3][32jp+16+dl]          at ((jp*4+G)*16+dl)*16
//   e4m3 K: 16-byte unit (j2, G, t)  = K[t][8(8j2+G)+0..7] , K[t][8(8j2+4+G)+0..7]
//   e4m3 V: 16-byte unit (jq, G, dl) = V[4G..4G+3][64jq+16u+dl], u = 0..3
//   e4m3 blocks start with a 128-byte header: fp32 sK[Hkv], fp32 sV[Hkv].
#include "pkv_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ u32x4 mk4(uint32_t a, uint32_t b, uint32_t c, uint32_t d) { return u32x4{a, b, c, d}; }
__device__ __forceinline__ u32x2 mk2(uint32_t a, uint32_t b) { return u32x2{a, b}; }

constexpr int T = 16;   // tokens per block the kernels are built for

__device__ __forceinline__ uint32_t pack_bf16_trunc(float lo, float hi) {
    // two fp32 -> packed bf16 by taking the upper halves (exact for values that
    // already fit bf16)
    return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
}

__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    f32x2 v = {lo, hi};
    bf16x2 b = __builtin_convertvector(v, bf16x2);
    return *reinterpret_cast<uint32_t *>(&b);
}

// 4 e4m3 codes in one word -> 4 bf16 in two words (exact)
__device__ __forceinline__ u32x2 fp8x4_to_bf16x4(uint32_t w) {
    f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false);
    f32x2 b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
    return mk2(pack_bf16_trunc(a[0], a[1]), pack_bf16_trunc(b[0], b[1]));
}

template <int D, int DT>
struct Tile {
    static constexpr int E = DT == PKV_BF16 ? 2 : 1;
    static constexpr int TILE_BYTES = T * D * E;           // one K or V tile
    static constexpr int NL = TILE_BYTES / 1024;           // 16-byte loads per lane per tile
    static constexpr int NK = D / 32;                      // QK^T MFMAs per page
    static constexpr int NV = D / 16;                      // d-tiles of the output
};

template <int D, int DT>
struct PageRegs {
    u32x4 k[Tile<D, DT>::NL];
    u32x4 v[Tile<D, DT>::NL];
    float sk, sv;
};

template <int D, int DT>
__device__ __forceinline__ void load_page(PageRegs<D, DT> &r, const AttnDesc &d, const int32_t *row, int page,
                                          int kvh, int lane) {
    uint32_t id = (uint32_t)row[page];
    if (id >= d.max_block_id) {          // never dereference an id outside the pool
        if (lane == 0) atomicOr(d.err, 1u);
        id = 0;
    }
    const uint32_t f = fastdiv_div(id, d.slots_div);
    const uint32_t s = id - f * d.slots_div.d;
    const uint8_t *blk = d.pool_base + (uint64_t)f * d.frame_bytes + (uint64_t)s * d.block_bytes;
    if (DT == PKV_E4M3) {
        const float *hdr = reinterpret_cast<const float *>(blk);
        r.sk = hdr[kvh];
        r.sv = hdr[d.Hkv + kvh];
        blk += PKV_FP8_HEADER;
    }
    const u32x4 *kp = reinterpret_cast<const u32x4 *>(blk + (size_t)kvh * 2 * Tile<D, DT>::TILE_BYTES) + lane;
    const u32x4 *vp = kp + Tile<D, DT>::TILE_BYTES / 16;
#pragma unroll
    for (int j = 0; j < Tile<D, DT>::NL; ++j) r.k[j] = __builtin_nontemporal_load(kp + j * 64);
#pragma unroll
    for (int j = 0; j < Tile<D, DT>::NL; ++j) r.v[j] = __builtin_nontemporal_load(vp + j * 64);
}

template <int D, int DT>
struct State {
    f32x4 acc[Tile<D, DT>::NV];   // out^T tiles: acc[jt][i] = out[16jt + 4G + i][head n]
    float m, l;                   // running max (log2 domain) and this lane's share of the sum
};

template <int D, int DT, bool TAIL>
__device__ __forceinline__ void process_page(State<D, DT> &st, const PageRegs<D, DT> &r, const bf16x8 *qf,
                                             float scale_log2, int valid /*tokens valid in this page*/, int G) {
    using TL = Tile<D, DT>;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    if (DT == PKV_BF16) {
#pragma unroll
        for (int j = 0; j < TL::NK; ++j) {
            u32x4 kv = r.k[j];
            s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<bf16x8 *>(&kv), qf[j], s, 0, 0, 0);
        }
    } else {
#pragma unroll
        for (int j2 = 0; j2 < TL::NL; ++j2) {
            const u32x4 kv = r.k[j2];
            const u32x2 a0 = fp8x4_to_bf16x4(kv.x), a1 = fp8x4_to_bf16x4(kv.y);
            const u32x2 b0 = fp8x4_to_bf16x4(kv.z), b1 = fp8x4_to_bf16x4(kv.w);
            u32x4 ka = mk4(a0.x, a0.y, a1.x, a1.y);
            u32x4 kb = mk4(b0.x, b0.y, b1.x, b1.y);
            s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<bf16x8 *>(&ka), qf[2 * j2], s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<bf16x8 *>(&kb), qf[2 * j2 + 1], s, 0, 0, 0);
        }
    }
    const float sc = DT == PKV_E4M3 ? scale_log2 * r.sk : scale_log2;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        s[i] *= sc;
        if (TAIL && 4 * G + i >= valid) s[i] = -INFINITY;
    }
    float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(st.m, mx);
    if (__any(m_new > st.m)) {            // wave-uniform: rescale only when some head's max moved
        const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
        st.l *= alpha;
#pragma unroll
        for (int jt = 0; jt < TL::NV; ++jt) st.acc[jt] *= alpha;
        st.m = m_new;
    }
    float p[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) p[i] = __builtin_amdgcn_exp2f(s[i] - st.m);
    st.l += (p[0] + p[1]) + (p[2] + p[3]);
    if (DT == PKV_E4M3) {
#pragma unroll
        for (int i = 0; i < 4; ++i) p[i] *= r.sv;
    }
    // P = hi + lo with both parts bf16: 16 significant bits reach the matrix unit
    const uint32_t h01 = pack_bf16_rne(p[0], p[1]), h23 = pack_bf16_rne(p[2], p[3]);
    const float l0 = p[0] - __uint_as_float(h01 << 16), l1 = p[1] - __uint_as_float(h01 & 0xffff0000u);
    const float l2 = p[2] - __uint_as_float(h23 << 16), l3 = p[3] - __uint_as_float(h23 & 0xffff0000u);
    u32x2 ph = mk2(h01, h23);
    u32x2 pl = mk2(pack_bf16_rne(l0, l1), pack_bf16_rne(l2, l3));
    const s16x4 phv = *reinterpret_cast<s16x4 *>(&ph), plv = *reinterpret_cast<s16x4 *>(&pl);
    // tokens past the context length may hold anything (even NaN): blank them
    uint32_t m01 = 0xffffffffu, m23 = 0xffffffffu;
    if (TAIL) {
        const int left = valid - 4 * G;
        m01 = left >= 2 ? 0xffffffffu : (left == 1 ? 0x0000ffffu : 0u);
        m23 = left >= 4 ? 0xffffffffu : (left == 3 ? 0x0000ffffu : 0u);
    }
#pragma unroll
    for (int jt = 0; jt < TL::NV; ++jt) {
        u32x2 a;
        if (DT == PKV_BF16) {
            const u32x4 vv = r.v[jt >> 1];
            a = (jt & 1) ? mk2(vv.z, vv.w) : mk2(vv.x, vv.y);
        } else {
            const u32x4 vv = r.v[jt >> 2];
            const uint32_t w = (jt & 3) == 0 ? vv.x : (jt & 3) == 1 ? vv.y : (jt & 3) == 2 ? vv.z : vv.w;
            a = fp8x4_to_bf16x4(w);
        }
        if (TAIL) {
            a.x &= m01;
            a.y &= m23;
        }
        const s16x4 av = *reinterpret_cast<s16x4 *>(&a);
        st.acc[jt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(av, phv, st.acc[jt], 0, 0, 0);
        st.acc[jt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(av, plv, st.acc[jt], 0, 0, 0);
    }
}

// Floats per split-K partial: g rows of D accumulators, then g maxima, then g sums.
__host__ __device__ inline int partial_floats(int g, int D) { return g * (D + 2); }

template <int D, int DT>
__device__ __forceinline__ void attn_item(const AttnDesc &d, int item) {
    using TL = Tile<D, DT>;
    const int lane = threadIdx.x;
    const int G = lane >> 4, n = lane & 15;
    const int kvh = item % d.Hkv;
    const int rest = item / d.Hkv;
    const int chunk = rest % d.max_chunks;
    const int seq = rest / d.max_chunks;
    int L = d.ctx_lens[seq];
    const int cap = d.row_stride * T;
    L = L < 0 ? 0 : (L > cap ? cap : L);
    const int n_pages = (L + T - 1) / T;
    const int C = d.chunk_pages;
    const int p0 = chunk * C;
    const int g = d.g;
    const int head = kvh * g + n;
    float *out_row = d.out + ((size_t)seq * d.Hq + head) * D;
    if (p0 >= n_pages) {
        if (chunk == 0 && n < g) {           // empty context: the row is defined as zero
#pragma unroll
            for (int jt = 0; jt < TL::NV; ++jt)
                *reinterpret_cast<f32x4 *>(out_row + 16 * jt + 4 * G) = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        return;
    }
    const int p1 = p0 + C < n_pages ? p0 + C : n_pages;
    const int n_chunks = (n_pages + C - 1) / C;
    const int32_t *row = d.table + (size_t)seq * d.row_stride;

    // q as the B operand: lane (G, n) holds q[head n][8(4j+G) .. +7] for each k-step j
    bf16x8 qf[TL::NK];
    {
        const uint16_t *qrow = d.q + ((size_t)seq * d.Hq + head) * D;
#pragma unroll
        for (int j = 0; j < TL::NK; ++j) {
            u32x4 v = mk4(0, 0, 0, 0);
            if (n < g) v = *reinterpret_cast<const u32x4 *>(qrow + 8 * (4 * j + G));
            qf[j] = *reinterpret_cast<bf16x8 *>(&v);
        }
    }

    State<D, DT> st;
#pragma unroll
    for (int jt = 0; jt < TL::NV; ++jt) st.acc[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
    st.m = -INFINITY;
    st.l = 0.f;

    const int last_valid = L - (n_pages - 1) * T;            // tokens in the last page, 1..16
    const bool tail_here = (p1 == n_pages) && last_valid < T;
    const int p_full_end = tail_here ? p1 - 1 : p1;          // pages [p0, p_full_end) are full

    PageRegs<D, DT> ra, rb;
    load_page<D, DT>(ra, d, row, p0, kvh, lane);
    int p = p0;
    // two pages per trip so the registers of the page in flight and the page in use
    // swap roles without copies
    for (; p + 1 < p_full_end; p += 2) {
        load_page<D, DT>(rb, d, row, p + 1, kvh, lane);
        process_page<D, DT, false>(st, ra, qf, d.scale_log2, T, G);
        if (p + 2 < p1) load_page<D, DT>(ra, d, row, p + 2, kvh, lane);
        process_page<D, DT, false>(st, rb, qf, d.scale_log2, T, G);
    }
    if (p < p_full_end) {                 // one full page left (ra holds it)
        if (p + 1 < p1) load_page<D, DT>(rb, d, row, p + 1, kvh, lane);
        process_page<D, DT, false>(st, ra, qf, d.scale_log2, T, G);
        ++p;
        if (p < p1) process_page<D, DT, true>(st, rb, qf, d.scale_log2, last_valid, G);
    } else if (p < p1) {                  // only the ragged page left (ra holds it)
        process_page<D, DT, true>(st, ra, qf, d.scale_log2, last_valid, G);
    }

    float l = st.l;
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    if (n >= g) return;
    if (n_chunks == 1) {
        const float inv = 1.0f / l;
#pragma unroll
        for (int jt = 0; jt < TL::NV; ++jt)
            *reinterpret_cast<f32x4 *>(out_row + 16 * jt + 4 * G) = st.acc[jt] * inv;
    } else {
        float *w = d.ws + (((size_t)seq * d.Hkv + kvh) * d.max_chunks + chunk) * partial_floats(g, D);
#pragma unroll
        for (int jt = 0; jt < TL::NV; ++jt)
            *reinterpret_cast<f32x4 *>(w + n * D + 16 * jt + 4 * G) = st.acc[jt];
        if (G == 0) {
            w[g * D + n] = st.m;
            w[g * D + g + n] = l;
        }
    }
}

__device__ __forceinline__ int find_model(const AttnGroup &grp, int item) {
    int mi = 0;
    for (int i = 1; i < grp.n; ++i)
        if (item >= grp.m[i].item_begin) mi = i;
    return mi;
}

__global__ __launch_bounds__(64) void k_attention(const AttnGroup grp) {
    const int gi = blockIdx.x;
    const int mi = find_model(grp, gi);
    const AttnDesc &d = grp.m[mi];
    const int item = gi - d.item_begin;
    if (d.dtype == PKV_BF16) {
        if (d.D == 128) attn_item<128, PKV_BF16>(d, item);
        else attn_item<64, PKV_BF16>(d, item);
    } else {
        if (d.D == 128) attn_item<128, PKV_E4M3>(d, item);
        else attn_item<64, PKV_E4M3>(d, item);
    }
}

// Split-K merge (online-softmax rule): with chunk maxima m_c, sums l_c and
// accumulators a_c,  M = max m_c,  out = sum_c 2^(m_c-M) a_c / sum_c 2^(m_c-M) l_c.
// One work-group per (sequence, query head), one lane per output element.
struct MergeGroup {
    int32_t row_begin[PKV_MAX_GROUP];   // first (seq, head) row of each model
    int32_t n;
};

__global__ void k_merge(const AttnGroup grp, const MergeGroup mg) {
    const int r = blockIdx.x;
    int mi = 0;
    for (int i = 1; i < mg.n; ++i)
        if (r >= mg.row_begin[i]) mi = i;
    const AttnDesc &d = grp.m[mi];
    const int rr = r - mg.row_begin[mi];
    const int seq = rr / d.Hq, head = rr % d.Hq;
    int L = d.ctx_lens[seq];
    const int cap = d.row_stride * T;
    L = L < 0 ? 0 : (L > cap ? cap : L);
    const int n_pages = (L + T - 1) / T;
    const int n_chunks = (n_pages + d.chunk_pages - 1) / d.chunk_pages;
    if (n_chunks <= 1) return;                      // written directly by the attention kernel
    const int g = d.g, D = d.D;
    const int kvh = head / g, n = head % g;
    const int pf = g * (D + 2);
    const float *w = d.ws + ((size_t)seq * d.Hkv + kvh) * d.max_chunks * pf;
    float M = -INFINITY;
    for (int c = 0; c < n_chunks; ++c) M = fmaxf(M, w[(size_t)c * pf + g * D + n]);
    const int t = threadIdx.x;
    if (t >= D) return;
    float num = 0.f, den = 0.f;
    for (int c = 0; c < n_chunks; ++c) {
        const float *wc = w + (size_t)c * pf;
        const float f = __builtin_amdgcn_exp2f(wc[g * D + n] - M);
        num += f * wc[n * D + t];
        den += f * wc[g * D + g + n];
    }
    d.out[((size_t)seq * d.Hq + head) * D + t] = num / den;
}

// kv_write: logical [n_tok][Hkv][D] -> the in-block operand layouts described above.
// One lane per (token, kv head, element); K and V handled together.
template <int DT>
__global__ void k_kv_write(AttnDesc d, const int32_t *row, int tok_begin, int n_tok, const uint8_t *k,
                           const uint8_t *v, const float *ks, const float *vs) {
    constexpr int E = DT == PKV_BF16 ? 2 : 1;
    const int D = d.D, Hkv = d.Hkv;
    const int64_t total = (int64_t)n_tok * Hkv * D;
    const int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int dd = (int)(idx % D);
    const int h = (int)((idx / D) % Hkv);
    const int ti = (int)(idx / ((int64_t)D * Hkv));
    const int tok = tok_begin + ti;
    const int page = tok / T, t = tok % T;
    const uint32_t id = (uint32_t)row[page];
    const uint32_t f = fastdiv_div(id, d.slots_div);
    const uint32_t s = id - f * d.slots_div.d;
    uint8_t *blk = const_cast<uint8_t *>(d.pool_base) + (uint64_t)f * d.frame_bytes + (uint64_t)s * d.block_bytes;
    if (DT == PKV_E4M3) {
        if (dd == 0) {
            const int srow = page - tok_begin / T;
            reinterpret_cast<float *>(blk)[h] = ks[(size_t)srow * Hkv + h];
            reinterpret_cast<float *>(blk)[Hkv + h] = vs[(size_t)srow * Hkv + h];
        }
        blk += PKV_FP8_HEADER;
    }
    const size_t tile = (size_t)T * D * E;
    uint8_t *kt = blk + (size_t)h * 2 * tile, *vt = kt + tile;
    const int G = t >> 2, e = t & 3;
    if (DT == PKV_BF16) {
        const size_t ko = ((size_t)((dd >> 3) * 16 + t)) * 8 + (dd & 7);
        const int jp = dd >> 5, half = (dd >> 4) & 1, dl = dd & 15;
        const size_t vo = ((size_t)((jp * 4 + G) * 16 + dl)) * 8 + half * 4 + e;
        reinterpret_cast<uint16_t *>(kt)[ko] = reinterpret_cast<const uint16_t *>(k)[idx];
        reinterpret_cast<uint16_t *>(vt)[vo] = reinterpret_cast<const uint16_t *>(v)[idx];
    } else {
        const int c8 = dd >> 3, j = c8 >> 2, Gk = c8 & 3, j2 = j >> 1, hf = j & 1;
        const size_t ko = ((size_t)((j2 * 4 + Gk) * 16 + t)) * 16 + hf * 8 + (dd & 7);
        const int jq = dd >> 6, u = (dd >> 4) & 3, dl = dd & 15;
        const size_t vo = ((size_t)((jq * 4 + G) * 16 + dl)) * 16 + u * 4 + e;
        kt[ko] = k[idx];
        vt[vo] = v[idx];
    }
}

}  // namespace

hipError_t pkv_launch_kv_write(const AttnDesc &d, int seq, int tok_begin, int n_tok, const void *k, const void *v,
                               const float *ks, const float *vs, int page_tokens, hipStream_t s) {
    (void)page_tokens;
    const int64_t total = (int64_t)n_tok * d.Hkv * d.D;
    if (total == 0) return hipSuccess;
    const int32_t *row = d.table + (size_t)seq * d.row_stride;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (d.dtype == PKV_BF16)
        hipLaunchKernelGGL(k_kv_write<PKV_BF16>, dim3(blocks), dim3(256), 0, s, d, row, tok_begin, n_tok,
                           (const uint8_t *)k, (const uint8_t *)v, ks, vs);
    else
        hipLaunchKernelGGL(k_kv_write<PKV_E4M3>, dim3(blocks), dim3(256), 0, s, d, row, tok_begin, n_tok,
                           (const uint8_t *)k, (const uint8_t *)v, ks, vs);
    return hipGetLastError();
}

hipError_t pkv_launch_attention(const AttnGroup &grp, hipStream_t s, hipEvent_t *ev) {
    int items = 0, rows = 0, maxD = 0;
    bool need_merge = false;
    MergeGroup mg;
    mg.n = grp.n;
    for (int i = 0; i < grp.n; ++i) {
        items += grp.m[i].n_items;
        mg.row_begin[i] = rows;
        rows += grp.m[i].batch * grp.m[i].Hq;
        if (grp.m[i].D > maxD) maxD = grp.m[i].D;
        if (grp.m[i].max_chunks > 1) need_merge = true;
    }
    if (items == 0) return hipSuccess;
    hipError_t e;
    if (ev && (e = hipEventRecord(ev[0], s)) != hipSuccess) return e;
    hipLaunchKernelGGL(k_attention, dim3(items), dim3(64), 0, s, grp);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (ev && (e = hipEventRecord(ev[1], s)) != hipSuccess) return e;
    if (need_merge && rows > 0) {
        hipLaunchKernelGGL(k_merge, dim3(rows), dim3(maxD), 0, s, grp, mg);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (ev && (e = hipEventRecord(ev[2], s)) != hipSuccess) return e;
    return hipSuccess;
}
