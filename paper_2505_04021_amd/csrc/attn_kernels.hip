// Paged GQA decode attention over the shared pool (gfx950 / CDNA4).
//
// Defines out = softmax(q K^T / sqrt(D)) V per sequence and query head, with K and V
// read through the sequence's block-table row (paper: Background, "KV cache and
// PagedAttention"; the balloon driver leaves attention semantics untouched, Sec. 4.2
// R4/D4).  The path is bound by HBM reads of K and V, each byte exactly once.
//
// Mapping to the hardware
//   * one wavefront (64 lanes) per work item; the pages of all (sequence, kv head)
//     pairs are laid end to end and cut into shares of equal expected time (pages plus
//     an allowance per segment, scaled by a weight per XCD), whatever the mix of
//     context lengths; where a share boundary
//     cuts a sequence, the wave that finishes it last merges the pieces with the
//     online-softmax rule inside the same kernel (partials and arrival counters sit in
//     uncached memory: no cache flush, no second launch);
//   * K and V tiles are stored inside a block in the lane order of the MFMA operands,
//     so each 16-byte global load is fully coalesced (64 lanes x 16 B = 1 KiB
//     contiguous) and lands directly in operand registers — no LDS round trip, no
//     shuffles between load and matrix op;
//   * the g query heads that share a kv head are padded to the 16 columns of one
//     MFMA tile: S[token][head] = K . q^T is a 16x16x32 bf16 MFMA per 32 elements of
//     head_dim; pages are taken two at a time, so out^T[d][head] += V^T . P contracts
//     over 32 tokens (4 + 4 per lane, one half from each page) in one 16x16x32 bf16
//     MFMA per 16 elements of head_dim, with P split into bf16 high and low parts (two
//     MFMAs) so that the probabilities keep 16 significant bits; accumulation is fp32;
//   * the softmax runs on the MFMA accumulator layout (lane = 4 tokens x 1 head, per
//     page): in-lane max / sum, then lane-permute swaps across the four lane rows,
//     once per page pair; no LDS in the streaming loop.
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

// Wave-uniform reads of data this kernel never writes (block tables, context
// lengths, the work plan, e4m3 scales): going through the constant address space
// makes them scalar loads, which are counted apart from the vector loads of K and V
// and so never force the KV pipeline to drain.
#define PKV_CONST(T_, p_) ((const T_ __attribute__((address_space(4))) *)(p_))

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

// 4 e4m3 codes in one word -> 4 bf16 in two words (exact): gfx950's packed conversion with a
// scale of one, two codes per instruction (checked against the fp32 route on all 2^16 code pairs)
__device__ __forceinline__ u32x2 fp8x4_to_bf16x4(uint32_t w) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false);
    bf16x2 b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true);
    return mk2(*reinterpret_cast<uint32_t *>(&a), *reinterpret_cast<uint32_t *>(&b));
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

// Block ids of a page pair.  They are read through the scalar cache one step before the
// loads that need them are issued, so the latency of this dependent access (block table
// -> address -> K/V load) is covered by the arithmetic of the step in between.
struct PairIds {
    uint32_t a, b;
};

__device__ __forceinline__ PairIds fetch_ids(const AttnDesc &d, const int32_t *row, int page) {
    const int last = d.row_stride - 1;
    const int ia = page < last ? page : last, ib = page + 1 < last ? page + 1 : last;
    PairIds ids;
    ids.a = (uint32_t)__builtin_amdgcn_readfirstlane(PKV_CONST(int32_t, row)[ia]);
    ids.b = (uint32_t)__builtin_amdgcn_readfirstlane(PKV_CONST(int32_t, row)[ib]);
    return ids;
}

// Issue the loads of one page (K tile, V tile) of one kv head.  Buffer loads with a
// per-page resource descriptor: a page beyond the chunk (live == false) gets a
// descriptor of zero records, so its loads return zeros without touching memory.
// That keeps every load of the software pipeline unconditional, which lets the
// compiler count outstanding loads exactly (s_waitcnt vmcnt(N) with N > 0) instead of
// draining the queue at each control-flow join.
template <int D, int DT>
__device__ __forceinline__ void load_page(PageRegs<D, DT> &r, const AttnDesc &d, uint32_t id, bool live, int kvh,
                                          int lane, uint32_t &bad) {
    using TL = Tile<D, DT>;
    if (id >= d.max_block_id) {          // never dereference an id outside the pool
        bad |= live ? 1u : 0u;           // reported once, after the last load (no store inside the loop)
        id = 0;
        live = false;                    // the page is skipped: frame 0 need not even be backed by memory
    }
    const uint32_t f = fastdiv_div(id, d.slots_div);
    const uint32_t s = id - f * d.slots_div.d;
    const uint8_t *blk = d.pool_base + (uint64_t)f * d.frame_bytes + (uint64_t)s * d.block_bytes;
    if (DT == PKV_E4M3) {
        // A dead page's id is whatever the table holds past the row's end: possibly a block of a
        // frame that was given back and, in an elastic pool, is no longer backed by memory.
        // Its header must not be read (the tile loads below are harmless: zero records).
        const float *hdr = reinterpret_cast<const float *>(live ? blk : reinterpret_cast<const uint8_t *>(d.safe));
        r.sk = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(PKV_CONST(float, hdr)[kvh])));
        r.sv = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(PKV_CONST(float, hdr)[d.Hkv + kvh])));
        if (!live) r.sk = r.sv = 0.f;
        blk += PKV_FP8_HEADER;
    }
    const uint8_t *tiles = blk + (size_t)kvh * 2 * TL::TILE_BYTES;
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(tiles), 0, live ? 2 * TL::TILE_BYTES : 0, 0x00020000);
    const int voff = lane * 16;
#pragma unroll
    for (int j = 0; j < TL::NL; ++j)
        r.k[j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff + j * 1024, 0, 2 /* non-temporal */);
#pragma unroll
    for (int j = 0; j < TL::NL; ++j)
        r.v[j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff + j * 1024, TL::TILE_BYTES, 2);
}

template <int D, int DT>
struct State {
    f32x4 acc[Tile<D, DT>::NV];   // out^T tiles: acc[jt][i] = out[16jt + 4G + i][head n]
    float m, l;                   // running max (log2 domain) and this lane's share of the sum
};

// Two consecutive pages of a piece travel and are processed together (32 tokens): one
// max / rescale step per 32 tokens and 16x16x32 MFMAs for the PV product.
template <int D, int DT>
struct PairRegs {
    PageRegs<D, DT> a, b;
};

template <int D, int DT>
__device__ __forceinline__ void load_pair(PairRegs<D, DT> &r, const AttnDesc &d, PairIds ids, bool live_a, bool live_b,
                                          int kvh, int lane, uint32_t &bad) {
    load_page<D, DT>(r.a, d, ids.a, live_a, kvh, lane, bad);
    load_page<D, DT>(r.b, d, ids.b, live_b, kvh, lane, bad);
}

// max over the four 16-lane rows of a wave (lanes l, l^16, l^32, l^48), in every lane.
// v_permlane32_swap exchanges the upper half of its first operand with the lower half of
// its second, v_permlane16_swap the odd rows of the first with the even rows of the
// second; fed the same value twice, the two results hold both partners of every lane.
// No LDS traffic, so the step does not wait on the scalar-load / LDS counter.
__device__ __forceinline__ float rows_max(float x) {
    typedef unsigned u2 __attribute__((ext_vector_type(2)));
    u2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// S[token][head] of one page: K (A operand, row = token) times q (B operand)
template <int D, int DT>
__device__ __forceinline__ f32x4 qk_page(const PageRegs<D, DT> &r, const bf16x8 *qf) {
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
    return s;
}

// V of one page for output tile jt as four bf16: V[4G..4G+3][16jt + (lane & 15)]
template <int D, int DT>
__device__ __forceinline__ u32x2 v_half(const PageRegs<D, DT> &r, int jt) {
    if (DT == PKV_BF16) {
        const u32x4 vv = r.v[jt >> 1];
        return (jt & 1) ? mk2(vv.z, vv.w) : mk2(vv.x, vv.y);
    }
    const u32x4 vv = r.v[jt >> 2];
    const uint32_t w = (jt & 3) == 0 ? vv.x : (jt & 3) == 1 ? vv.y : (jt & 3) == 2 ? vv.z : vv.w;
    return fp8x4_to_bf16x4(w);
}

// Probabilities reach the matrix unit as bf16: as hi + lo (16 significant bits, two products)
// wherever the second product is free or the cache is bf16.  The exception is prefill (bound by
// arithmetic, not by memory) on an e4m3 cache: its values carry 4 significant bits, one bf16
// probability (8 bits, error 2^-9) is already 32 times finer than the V it multiplies, and the
// second product is left out (measured error then ~4e-3 of a row's largest output against a bar of
// 2e-2; 16 % less time).
template <int DT, bool PREFILL>
__device__ __forceinline__ constexpr bool p_has_lo() {
    return DT == PKV_BF16 || !PREFILL;
}

// bf16 hi + lo of four probabilities: 16 significant bits reach the matrix unit
__device__ __forceinline__ void split_p(const float *p, u32x2 &hi, u32x2 &lo) {
    const uint32_t h01 = pack_bf16_rne(p[0], p[1]), h23 = pack_bf16_rne(p[2], p[3]);
    const float l0 = p[0] - __uint_as_float(h01 << 16), l1 = p[1] - __uint_as_float(h01 & 0xffff0000u);
    const float l2 = p[2] - __uint_as_float(h23 << 16), l3 = p[3] - __uint_as_float(h23 & 0xffff0000u);
    hi = mk2(h01, h23);
    lo = mk2(pack_bf16_rne(l0, l1), pack_bf16_rne(l2, l3));
}

// Largest of three in one instruction.  Written out because the compiler puts a quieting instruction in
// front of every matrix-unit result that it takes a maximum of.
__device__ __forceinline__ float max3(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// How far (in powers of two) a column's maximum may run ahead of the reference point of its
// exponentials before a softmax step moves that point and rescales the column's sums.  The reference
// point need not be the true maximum, only near it: results are the same up to rounding (probabilities
// up to 2^kRescaleSlack instead of 1, numerator and denominator alike), and the 32 multiplications of a
// rescale become rare.
constexpr float kRescaleSlack = 8.f;

// One online-softmax step over the 32 tokens of a page pair.  valid_a is 1..16,
// valid_b 0..16 (0: the pair has no second page; its registers hold zeros).
// TAIL: 0 = whether the pair needs masks is decided at run time inside (one code path with
// selects: right for the memory-bound decode kernel), 1 = the caller knows it needs none,
// 2 = the caller knows it needs them (the prefill kernel branches, its bound is vector ALU work).
template <int D, int DT, bool CAUSAL, int TAIL = 0>
__device__ __forceinline__ void process_pair(State<D, DT> &st, const PairRegs<D, DT> &r, const bf16x8 *qf,
                                             float scale_log2, int valid_a, int valid_b, int G, int lim_a = 0,
                                             bool causal = false) {
    using TL = Tile<D, DT>;
    const bool tail = TAIL == 1 ? false : (TAIL == 2 ? true : (valid_a < T || valid_b < T || (CAUSAL && causal)));
    f32x4 sa = qk_page<D, DT>(r.a, qf);
    f32x4 sb = qk_page<D, DT>(r.b, qf);
    const float sca = DT == PKV_E4M3 ? scale_log2 * r.a.sk : scale_log2;
    const float scb = DT == PKV_E4M3 ? scale_log2 * r.b.sk : scale_log2;
    float s[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        s[i] = sa[i] * sca;
        s[4 + i] = sb[i] * scb;
        if (tail) {                                        // select, so a NaN logit of a dead token cannot leak
            const int la = CAUSAL && lim_a < valid_a ? lim_a : valid_a;
            const int lb = CAUSAL && lim_a - T < valid_b ? lim_a - T : valid_b;
            if (4 * G + i >= la) s[i] = -INFINITY;
            if (4 * G + i >= lb) s[4 + i] = -INFINITY;
        }
    }
    float mx = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
    mx = rows_max(mx);
    const float m_new = fmaxf(st.m, mx);
    // wave-uniform: the reference point of the exponentials moves, and the sums are rescaled, only when some
    // column's maximum has run ahead of it by more than kRescaleSlack (probabilities stay below 2^kRescaleSlack)
    if (__any(m_new > st.m + kRescaleSlack)) {
        // a column that has seen no token yet (prefill tiles only) has m = -inf on both sides
        const float alpha = CAUSAL && TAIL != 1 && m_new == -INFINITY ? 1.0f : __builtin_amdgcn_exp2f(st.m - m_new);
        st.l *= alpha;
#pragma unroll
        for (int jt = 0; jt < TL::NV; ++jt) st.acc[jt] *= alpha;
        st.m = m_new;
    }
    float p[8];
    // (a pair without masks leaves every column with a finite maximum)
    const float m_ref = CAUSAL && TAIL != 1 && st.m == -INFINITY ? 0.f : st.m;     // then every s is -inf and every p is 0
#pragma unroll
    for (int i = 0; i < 8; ++i) p[i] = __builtin_amdgcn_exp2f(s[i] - m_ref);
    st.l += ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
    if (DT == PKV_E4M3) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            p[i] *= r.a.sv;
            p[4 + i] *= r.b.sv;
        }
    }
    // B operand of the PV product: lane (G, head) holds P for tokens 4G..4G+3 of page a, then of page b
    u32x2 ha, la, hb, lb;
    split_p(p, ha, la);
    split_p(p + 4, hb, lb);
    u32x4 ph = mk4(ha.x, ha.y, hb.x, hb.y), pl = mk4(la.x, la.y, lb.x, lb.y);
    const bf16x8 phv = *reinterpret_cast<bf16x8 *>(&ph), plv = *reinterpret_cast<bf16x8 *>(&pl);
    // tokens past the context length may hold anything (even NaN): blank their V
    uint32_t ma01 = 0xffffffffu, ma23 = 0xffffffffu, mb01 = 0xffffffffu, mb23 = 0xffffffffu;
    if (tail) {
        const int la_ = valid_a - 4 * G, lb_ = valid_b - 4 * G;
        ma01 = la_ >= 2 ? 0xffffffffu : (la_ == 1 ? 0x0000ffffu : 0u);
        ma23 = la_ >= 4 ? 0xffffffffu : (la_ == 3 ? 0x0000ffffu : 0u);
        mb01 = lb_ >= 2 ? 0xffffffffu : (lb_ == 1 ? 0x0000ffffu : 0u);
        mb23 = lb_ >= 4 ? 0xffffffffu : (lb_ == 3 ? 0x0000ffffu : 0u);
    }
#pragma unroll
    for (int jt = 0; jt < TL::NV; ++jt) {
        // A operand: V^T, row = output element 16jt + (lane & 15), k = the same eight tokens
        const u32x2 va = v_half<D, DT>(r.a, jt), vb = v_half<D, DT>(r.b, jt);
        u32x4 vv = tail ? mk4(va.x & ma01, va.y & ma23, vb.x & mb01, vb.y & mb23) : mk4(va.x, va.y, vb.x, vb.y);
        const bf16x8 av = *reinterpret_cast<bf16x8 *>(&vv);
        st.acc[jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, phv, st.acc[jt], 0, 0, 0);
        if (p_has_lo<DT, CAUSAL>()) st.acc[jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, plv, st.acc[jt], 0, 0, 0);
    }
}

// The two halves of process_pair for a pair that needs no masks, for callers that work on
// several tiles of queries at once (prefill): with the halves of all tiles in one straight
// line of code the scheduler can overlap the matrix instructions of one tile with the
// softmax arithmetic of another.
template <int D, int DT>
__device__ __forceinline__ void pair_qk(const PairRegs<D, DT> &r, const bf16x8 *qf, f32x4 &sa, f32x4 &sb) {
    sa = qk_page<D, DT>(r.a, qf);
    sb = qk_page<D, DT>(r.b, qf);
}

// The same for two tiles of queries at once (bf16 caches): four independent accumulation chains (two
// pages x two tiles), written round-robin so that no matrix instruction waits for the one before it.
template <int D>
__device__ __forceinline__ void pair_qk2(const PairRegs<D, PKV_BF16> &r, const bf16x8 *q0, const bf16x8 *q1, f32x4 *sa, f32x4 *sb) {
    using TL = Tile<D, PKV_BF16>;
    f32x4 a0 = {0.f, 0.f, 0.f, 0.f}, b0 = a0, a1 = a0, b1 = a0;
#pragma unroll
    for (int j = 0; j < TL::NK; ++j) {
        u32x4 ka = r.a.k[j], kb = r.b.k[j];
        const bf16x8 kav = *reinterpret_cast<bf16x8 *>(&ka), kbv = *reinterpret_cast<bf16x8 *>(&kb);
        a0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kav, q0[j], a0, 0, 0, 0);
        b0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kbv, q0[j], b0, 0, 0, 0);
        a1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kav, q1[j], a1, 0, 0, 0);
        b1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kbv, q1[j], b1, 0, 0, 0);
    }
    sa[0] = a0; sb[0] = b0; sa[1] = a1; sb[1] = b1;
}

template <int D, int DT>
__device__ __forceinline__ void pair_softmax(State<D, DT> &st, const PairRegs<D, DT> &r, f32x4 sa, f32x4 sb, float scale_log2,
                                             bf16x8 &phv, bf16x8 &plv) {
    using TL = Tile<D, DT>;
    const float sca = DT == PKV_E4M3 ? scale_log2 * r.a.sk : scale_log2;
    const float scb = DT == PKV_E4M3 ? scale_log2 * r.b.sk : scale_log2;
    float s[8];
    float mx;
    if (DT == PKV_E4M3) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            s[i] = sa[i] * sca;
            s[4 + i] = sb[i] * scb;
        }
        mx = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
    } else {
        // one positive scale for all: the maximum is taken on the raw scores and scaled once, and the
        // scale of each score is folded into the argument of its exponential below
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            s[i] = sa[i];
            s[4 + i] = sb[i];
        }
        mx = scale_log2 * max3(max3(s[0], s[1], s[2]), max3(s[3], s[4], s[5]), max3(s[6], s[7], s[0]));
    }
    // The reference point of the exponentials need not be the true maximum, only near it: it moves (and
    // the sums are rescaled) when some column's maximum has grown by more than kRescaleSlack, so that
    // probabilities stay below 2^kRescaleSlack.  Wave-uniform.
    mx = rows_max(mx);
    const float m_new = fmaxf(st.m, mx);
    if (__any(m_new > st.m + kRescaleSlack)) {
        const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
        st.l *= alpha;
#pragma unroll
        for (int jt = 0; jt < TL::NV; ++jt) st.acc[jt] *= alpha;
        st.m = m_new;
    }
    float p[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
        p[i] = __builtin_amdgcn_exp2f(DT == PKV_E4M3 ? s[i] - st.m : __builtin_fmaf(s[i], scale_log2, -st.m));
    st.l += ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
    if (DT == PKV_E4M3) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            p[i] *= r.a.sv;
            p[4 + i] *= r.b.sv;
        }
    }
    u32x2 ha, la, hb, lb;
    split_p(p, ha, la);
    split_p(p + 4, hb, lb);
    u32x4 ph = mk4(ha.x, ha.y, hb.x, hb.y), pl = mk4(la.x, la.y, lb.x, lb.y);
    phv = *reinterpret_cast<bf16x8 *>(&ph);
    plv = *reinterpret_cast<bf16x8 *>(&pl);
}

template <int D, int DT>
__device__ __forceinline__ void pair_accumulate(State<D, DT> &st, const PairRegs<D, DT> &r, bf16x8 phv, bf16x8 plv) {
    using TL = Tile<D, DT>;
#pragma unroll
    for (int jt = 0; jt < TL::NV; ++jt) {
        const u32x2 va = v_half<D, DT>(r.a, jt), vb = v_half<D, DT>(r.b, jt);
        u32x4 vv = mk4(va.x, va.y, vb.x, vb.y);
        const bf16x8 av = *reinterpret_cast<bf16x8 *>(&vv);
        st.acc[jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, phv, st.acc[jt], 0, 0, 0);
        if (p_has_lo<DT, true>()) st.acc[jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, plv, st.acc[jt], 0, 0, 0);
    }
}

// The same with the operands of the accumulation already assembled (bf16 tiles read from LDS in
// halves: vop[jt] = the V half of page a and the V half of page b for output tile jt).
template <int D, int DT>
__device__ __forceinline__ void pair_accumulate_ops(State<D, DT> &st, const u32x4 *vop, bf16x8 phv, bf16x8 plv) {
    using TL = Tile<D, DT>;
#pragma unroll
    for (int jt = 0; jt < TL::NV; ++jt) {
        u32x4 vv = vop[jt];
        const bf16x8 av = *reinterpret_cast<bf16x8 *>(&vv);
        st.acc[jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, phv, st.acc[jt], 0, 0, 0);
        if (p_has_lo<DT, true>()) st.acc[jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, plv, st.acc[jt], 0, 0, 0);
    }
}

// Floats per split-K partial: g rows of D accumulators, then g maxima, then g sums.
__host__ __device__ inline int partial_floats(int g, int D) { return g * (D + 2); }

constexpr int FLIGHT_KIB_2WAVES = 16;      // bytes in flight per wave, two waves per SIMD
// Page pairs resident per wave: one in use, the rest in flight.  In the form with two waves per
// SIMD every shape keeps the same number of bytes in flight (FLIGHT_KIB_2WAVES), small pages
// through a deeper ring; otherwise waves of a small-page model would fall behind the others in
// a grouped launch.
template <int D, int DT, int FLIGHT_KIB = FLIGHT_KIB_2WAVES>
struct Ring {
    static constexpr int PAIR_BYTES = 4 * Tile<D, DT>::TILE_BYTES;        // K and V tiles of two pages
    static constexpr int N = 1 + (FLIGHT_KIB * 1024 + PAIR_BYTES - 1) / PAIR_BYTES;
};
// The second form of the kernel: one wave per SIMD, the host launching only as many waves as it
// takes to keep the memory system busy (512 for bf16 pages of 8 KiB).  A wave alone on its SIMD
// turns a page pair over in 0.7-1.1 us whatever it has in flight, so one pair in use and one
// travelling is all the ring needs (8 KiB covers a pair of every shape but bf16 with 128-wide
// heads, whose pair of 16 KiB is the one in flight anyway); more bytes outstanding only lengthen
// the queues in front of the memory channels, and the launch as a whole gets slower.
constexpr int FLIGHT_KIB_1WAVE = 8;
constexpr int MAX_PIECES = 64;   // pieces of one (sequence, kv head) the merge stages in LDS

// A row of a launch.  In a decode step it is a sequence with its one new query token.  In a
// prefill launch it is a tile of consecutive query tokens of a sequence's chunk (as many as
// fit the 16 MFMA columns together with the g heads of a kv head): `seq` is the sequence,
// `q0` the first of the tile's rows in the packed q and out arrays, `ntok` their number,
// and `back` how many chunk tokens follow the tile, so that the tile's last token sees
// ctx_lens[seq] - back tokens.
struct RowInfo {
    int seq, q0, back, ntok;
};

__device__ __forceinline__ RowInfo row_info_uniform(const AttnDesc &d, int row) {
    if (!d.vmap) return RowInfo{row, row, 0, 1};
    const int32_t *v = reinterpret_cast<const int32_t *>(d.vmap + row);
    return RowInfo{__builtin_amdgcn_readfirstlane(PKV_CONST(int32_t, v)[0]), __builtin_amdgcn_readfirstlane(PKV_CONST(int32_t, v)[1]),
                   __builtin_amdgcn_readfirstlane(PKV_CONST(int32_t, v)[2]), __builtin_amdgcn_readfirstlane(PKV_CONST(int32_t, v)[3])};
}

__device__ __forceinline__ int ctx_clamped(const AttnDesc &d, int seq) {
    int L = PKV_CONST(int32_t, d.ctx_lens)[seq];
    const int cap = (d.row_len ? PKV_CONST(int32_t, d.row_len)[seq] : d.row_stride) * T;
    return L < 0 ? 0 : (L > cap ? cap : L);
}

// Length a segment is given on the line the shares are cut from: its pages plus a fixed
// allowance for what every segment costs besides its pages (the turn it does not fill,
// the gap in the stream at its boundary, writing its result), at least 1 so that an
// empty sequence still has an owner who writes its zero row.
__device__ __forceinline__ int planned(const AttnDesc &d, int n_pages) {
    const int pl = n_pages + d.seg_cost;
    return pl > 0 ? pl : 1;
}

// A piece: the pages [pb, pe) of one (sequence, kv head) segment that fall into this
// wave's share.  All fields are wave-uniform.
struct Piece {
    int valid;                  // 0 past the end of the share
    int seq, kvh;
    int P;                      // planned pages of all earlier sequences
    int L, n_pages, pl;         // context length, its pages, planned pages (>= 1)
    int pb, pe;                 // page range of the piece inside the segment
    uint32_t g0;                // where the segment starts on the line of page units
};

__device__ __forceinline__ void piece_set_seq(Piece &pc, const AttnDesc &d, int seq, int P) {
    pc.seq = seq;
    pc.P = P;
    pc.L = seq < d.batch ? __builtin_amdgcn_readfirstlane(ctx_clamped(d, seq < d.batch ? seq : 0)) : 0;
    pc.n_pages = (pc.L + T - 1) / T;
    pc.pl = planned(d, pc.n_pages);
}

// clip segment (seq, kvh) against the share [gbeg, gend)
__device__ __forceinline__ void piece_clip(Piece &pc, const AttnDesc &d, uint32_t gbeg, uint32_t gend) {
    pc.g0 = (uint32_t)pc.P * d.Hkv + (uint32_t)pc.kvh * pc.pl;
    pc.valid = (pc.seq < d.batch && pc.g0 < gend) ? 1 : 0;
    pc.pb = gbeg > pc.g0 ? (int)(gbeg - pc.g0) : 0;
    pc.pe = gend - pc.g0 < (uint32_t)pc.pl ? (int)(gend - pc.g0) : pc.pl;
    // the allowance past the last page holds no work; an empty sequence has the one unit [0, 1)
    const int real = pc.n_pages > 0 ? pc.n_pages : 1;
    pc.pe = pc.pe < real ? pc.pe : real;
}

__device__ __forceinline__ Piece piece_next(const Piece &c, const AttnDesc &d, uint32_t gbeg, uint32_t gend) {
    Piece nx = c;
    if (c.kvh + 1 < d.Hkv) {
        nx.kvh = c.kvh + 1;
    } else {
        nx.kvh = 0;
        piece_set_seq(nx, d, c.seq + 1, c.P + c.pl);
    }
    piece_clip(nx, d, gbeg, gend);
    return nx;
}

// Which (query token of the row, head of the kv head's group) an MFMA column stands for.
struct Column {
    int tok, head;      // column n = tok * g + head
};

__device__ __forceinline__ Column column_of(const AttnDesc &d, int n) {
    const int tok = n / d.g;
    return Column{tok, n - tok * d.g};
}

// q as the B operand: lane (G, n) holds q[column n][8(4j+G) .. +7] for each k-step j
template <int D>
__device__ __forceinline__ void load_q(bf16x8 *qf, const AttnDesc &d, const RowInfo &ri, int kvh, int lane, Column col) {
    const int G = lane >> 4, n = lane & 15;
    const uint16_t *qrow = d.q + ((size_t)(ri.q0 + col.tok) * d.Hq + kvh * d.g + col.head) * D;
    const bool live = n < d.cols && col.tok < ri.ntok;
#pragma unroll
    for (int j = 0; j < D / 32; ++j) {
        u32x4 v = mk4(0, 0, 0, 0);
        if (live) v = *reinterpret_cast<const u32x4 *>(qrow + 8 * (4 * j + G));
        qf[j] = *reinterpret_cast<bf16x8 *>(&v);
    }
}

// What is left to do for a piece whose segment is shared with other waves: once the
// arrival count is back, the wave that came last merges.
struct Pending {
    int valid, seq, kvh;
    uint32_t k0, k1, arrived;
};

// online-softmax merge of the pieces of one segment: M = max m_c,
// out = sum_c 2^(m_c-M) a_c / sum_c 2^(m_c-M) l_c.  Piece c of the segment sits in
// share k0 + c: slot b of that share for c = 0, slot a otherwise.
// The partials come from uncached memory, so the cost is memory round trips: each lane
// owns EPL groups of four consecutive output elements and fetches the accumulators of
// 32 / EPL pieces per trip; the maxima and sums of all pieces travel with the first trip
// and are staged in LDS.
template <int D, int EPL>
__device__ __forceinline__ void merge_rows(const AttnDesc &d, const Pending &pd, int lane, float *s_m, float *s_l,
                                           const float *base, int n_pc) {
    constexpr int D4 = D / 4;
    constexpr int PB = 32 / EPL;                      // pieces per trip
    const int g = d.cols, pf = partial_floats(g, D);  // g: columns (query token, head) of a partial
    const int E = g * D4;
    const RowInfo ri = row_info_uniform(d, pd.seq);
    int hn[EPL], x[EPL];
#pragma unroll
    for (int k = 0; k < EPL; ++k) {
        const int e = lane + 64 * k;
        const int ee = e < E ? e : E - 1;             // idle lanes shadow a valid element
        hn[k] = ee / D4;
        x[k] = ee - hn[k] * D4;
    }
    // first trip: the accumulators of the first PB pieces travel together with all maxima and sums
    f32x4 v[PB][EPL];
#pragma unroll
    for (int u = 0; u < PB; ++u) {
        const int c = u < n_pc ? u : n_pc - 1;
        const float *wc = base + (size_t)(2 * c + (c == 0 ? 1 : 0)) * pf;
#pragma unroll
        for (int k = 0; k < EPL; ++k) v[u][k] = *reinterpret_cast<const f32x4 *>(wc + hn[k] * D + 4 * x[k]);
    }
    for (int i = lane; i < n_pc * g; i += 64) {
        const int c = i / g, h = i - c * g;
        const float *wc = base + (size_t)(2 * c + (c == 0 ? 1 : 0)) * pf + g * D;
        s_m[i] = wc[h];
        s_l[i] = wc[g + h];
    }
    __builtin_amdgcn_wave_barrier();     // one wave per work-group: program order is enough
    float M[EPL], den[EPL];
    f32x4 num[EPL];
#pragma unroll
    for (int k = 0; k < EPL; ++k) {
        float mm = -INFINITY;
        for (int c = 0; c < n_pc; ++c) mm = fmaxf(mm, s_m[c * g + hn[k]]);
        M[k] = mm;
        den[k] = 0.f;
        num[k] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    for (int c0 = 0; c0 < n_pc; c0 += PB) {
        if (c0 > 0) {
#pragma unroll
            for (int u = 0; u < PB; ++u) {
                const int c = c0 + u < n_pc ? c0 + u : n_pc - 1;
                const float *wc = base + (size_t)(2 * c + (c == 0 ? 1 : 0)) * pf;
#pragma unroll
                for (int k = 0; k < EPL; ++k) v[u][k] = *reinterpret_cast<const f32x4 *>(wc + hn[k] * D + 4 * x[k]);
            }
        }
#pragma unroll
        for (int u = 0; u < PB; ++u) {
            if (c0 + u < n_pc) {
#pragma unroll
                for (int k = 0; k < EPL; ++k) {
                    const float f = __builtin_amdgcn_exp2f(s_m[(c0 + u) * g + hn[k]] - M[k]);
                    den[k] += f * s_l[(c0 + u) * g + hn[k]];
                    num[k] += f * v[u][k];
                }
            }
        }
    }
#pragma unroll
    for (int k = 0; k < EPL; ++k) {
        const Column col = column_of(d, hn[k]);
        if (lane + 64 * k < E && col.tok < ri.ntok)
            *reinterpret_cast<f32x4 *>(d.out + ((size_t)(ri.q0 + col.tok) * d.Hq + pd.kvh * d.g + col.head) * D + 4 * x[k]) =
                num[k] * (1.0f / den[k]);
    }
    __builtin_amdgcn_wave_barrier();
}

template <int D>
__device__ __forceinline__ void merge_segment(const AttnDesc &d, const Pending &pd, int lane, float *s_m, float *s_l) {
    const int g = d.cols, pf = partial_floats(g, D);
    const int n_pc = (int)(pd.k1 - pd.k0) + 1;
    const float *base = d.ws + (size_t)(2 * pd.k0) * pf;
    const int groups = (g * (D / 4) + 63) / 64;       // element groups per lane
    if (groups <= 1) merge_rows<D, 1>(d, pd, lane, s_m, s_l, base, n_pc);
    else if (groups <= 2) merge_rows<D, 2>(d, pd, lane, s_m, s_l, base, n_pc);
    else if (groups <= 4) merge_rows<D, 4>(d, pd, lane, s_m, s_l, base, n_pc);
    else merge_rows<D, 8>(d, pd, lane, s_m, s_l, base, n_pc);
}

// Work split ("stream-K" over pages): the (sequence, kv head) segments of a model are
// laid end to end, a segment being the pages of one sequence for one kv head; the
// resulting line of W page units is cut into equal shares, one per wave.  A wave's
// share may end inside a segment and start inside another: such pieces leave a partial
// (accumulators, max, sum) in uncached memory, and the wave that completes a segment
// last merges its pieces with the online-softmax rule.  Segments that lie inside one
// share are finished directly.  Every wave derives the split from ctx_lens itself, so
// the split follows the real context lengths and needs no host-side plan.
//
// Inside a share the pages of consecutive pieces form ONE stream through the register
// ring: pages travel and are processed in pairs (32 tokens), work proceeds in turns of
// RING pairs, every piece is padded to whole turns with dead pages (no traffic, no
// math), and during the last turn of a piece the loads already fetch the first pairs of
// the next piece.
// Where the shares of the work items begin on the line of page units.  Items come in
// blocks of eight (one per XCD); a block spans 8 * share units and is cut at
// cum[j] / 65536 of its length (cum[0] = 0, cum[8] = 65536), or evenly without weights.
constexpr uint32_t WEIGHTED_SHARE_MIN = 16;     // below this, uneven cuts could leave a share empty
struct Cut {
    uint32_t share;
    const uint32_t *cum;        // kernel-argument memory, or NULL for even cuts

    __device__ __forceinline__ uint32_t begin(uint32_t item) const {
        if (!cum) return item * share;
        const uint32_t blk = item >> 3, j = item & 7u;
        return blk * 8u * share + (uint32_t)(((uint64_t)(8u * share) * PKV_CONST(uint32_t, cum)[j]) >> 16);
    }
    // the item whose share holds line position x
    __device__ __forceinline__ uint32_t index(uint32_t x) const {
        if (!cum) return x / share;
        const uint32_t s8 = 8u * share, blk = x / s8, rem = x - blk * s8;
        uint32_t j = 0;
#pragma unroll
        for (uint32_t t = 1; t < 8; ++t)
            j += rem >= (uint32_t)(((uint64_t)s8 * PKV_CONST(uint32_t, cum)[t]) >> 16) ? 1u : 0u;
        return blk * 8u + j;
    }
};


// CACHED: the partials and arrival counters sit in ordinary (cached) device memory instead of
// uncached memory.  The L2 caches of the eight XCDs are not coherent with each other for such
// memory, so the hand-over of a partial follows the memory model by the book: partial stores,
// release fence, arrival atomic (agent scope) on the writer's side; arrival atomic, acquire fence,
// partial loads on the merger's side.
template <int D, int DT, int FLIGHT_KIB = FLIGHT_KIB_2WAVES, bool CACHED = false>
__device__ __forceinline__ void attn_wave(const AttnDesc &d, const AttnTune &w, int item, float *s_m, float *s_l) {
    using TL = Tile<D, DT>;
    const int lane = threadIdx.x;
    __builtin_amdgcn_s_setprio(3);      // from the first instruction: a wave still setting up must not wait behind streaming ones
    const int G = lane >> 4, n = lane & 15;
    const int g = d.cols, Hkv = d.Hkv, B = d.batch;   // g: columns in use, (query tokens of a row) x (heads of a kv head)
    const Column col = column_of(d, n);
    const uint64_t t_begin = w.stat ? wall_clock64() : 0;

    // --- planned pages per sequence, prefix sums across the wave.  Batches of up to
    // 64 * LINE_REGS sequences keep every context length in registers, so that finding
    // the first segment costs no further memory access.
    constexpr int LINE_REGS = 4;
    const int K = (B + 63) >> 6;                    // sequences per lane
    int Lc[LINE_REGS];
    int my_sum = 0, my_max = 0;
#pragma unroll
    for (int k = 0; k < LINE_REGS; ++k) {
        const int sq = lane * K + k;
        Lc[k] = (k < K && sq < B) ? ctx_clamped(d, sq) : -1;
    }
    if (K <= LINE_REGS) {
#pragma unroll
        for (int k = 0; k < LINE_REGS; ++k) {
            if (Lc[k] >= 0) {
                const int np = (Lc[k] + T - 1) / T;
                const int pl = planned(d, np);
                my_sum += pl;
                my_max = pl > my_max ? pl : my_max;
            }
        }
    } else {
        for (int k = 0; k < K; ++k) {
            const int sq = lane * K + k;
            if (sq < B) {
                const int np = (ctx_clamped(d, sq) + T - 1) / T;
                const int pl = planned(d, np);
                my_sum += pl;
                my_max = pl > my_max ? pl : my_max;
            }
        }
    }
    int incl = my_sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o);
        if (lane >= o) incl += v;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const int v = __shfl_xor(my_max, o);
        my_max = v > my_max ? v : my_max;
    }
    const int total = __builtin_amdgcn_readlane(incl, 63);
    const uint32_t W = (uint32_t)total * (uint32_t)Hkv;
    // Shares: equal in the mean, but never so small that a segment falls into more pieces
    // than the merge can stage.  Eight consecutive items run on the eight XCDs (work-groups
    // are dealt to them in turn), and XCDs do not all get the same memory bandwidth; so a
    // block of eight shares is cut at the caller's cumulative weights instead of evenly.
    uint32_t share = (W + (uint32_t)d.n_items - 1) / (uint32_t)d.n_items;
    const uint32_t floor_share = ((uint32_t)my_max + (MAX_PIECES - 24) - 1) / (MAX_PIECES - 24);
    share = share < floor_share ? floor_share : share;
    share = share < (uint32_t)d.min_share ? (uint32_t)d.min_share : share;
    share = (uint32_t)__builtin_amdgcn_readfirstlane((int)share);
    const Cut cut = Cut{share, (share >= WEIGHTED_SHARE_MIN && d.weighted) ? w.cum : nullptr};
    const uint32_t gbeg = cut.begin((uint32_t)item);
    uint32_t gend = cut.begin((uint32_t)item + 1);
    if (gbeg >= W) return;
    gend = gend < W ? gend : W;

    // --- which segment holds line position x: the lane whose sequences span x walks them (from
    // registers for batches that fit there)
    auto locate = [&](uint32_t x, int &seq, int &P, int &L) {
        const uint32_t lo = (uint32_t)(incl - my_sum) * Hkv, hi = (uint32_t)incl * Hkv;
        const unsigned long long own = __ballot(lo <= x && x < hi);
        const int owner = __ffsll(own) - 1;
        int fs = 0, fp = incl - my_sum, fl = 0;     // sequence, pages before it, its context length
        if (K <= LINE_REGS) {
            bool found = false;
#pragma unroll
            for (int k = 0; k < LINE_REGS; ++k) {
                if (!found && Lc[k] >= 0) {
                    const int np = (Lc[k] + T - 1) / T;
                    const int pl = planned(d, np);
                    if ((uint32_t)(fp + pl) * Hkv <= x) fp += pl;
                    else { fs = lane * K + k; fl = Lc[k]; found = true; }
                }
            }
        } else {
            for (int k = 0; k < K; ++k) {           // only the owner's walk matters
                const int sq = lane * K + k;
                if (sq < B) {
                    const int L1 = ctx_clamped(d, sq);
                    const int np = (L1 + T - 1) / T;
                    const int pl = planned(d, np);
                    if ((uint32_t)(fp + pl) * Hkv <= x) fp += pl; else { fs = sq; fl = L1; break; }
                }
            }
        }
        seq = __builtin_amdgcn_readfirstlane(__shfl(fs, owner));
        P = __builtin_amdgcn_readfirstlane(__shfl(fp, owner));
        L = __builtin_amdgcn_readfirstlane(__shfl(fl, owner));
    };
    auto piece_at = [&](uint32_t x) {
        Piece pc;
        locate(x, pc.seq, pc.P, pc.L);
        pc.n_pages = (pc.L + T - 1) / T;
        pc.pl = planned(d, pc.n_pages);
        pc.kvh = (int)((x - (uint32_t)pc.P * Hkv) / (uint32_t)pc.pl);
        piece_clip(pc, d, gbeg, gend);
        return pc;
    };

    // --- the first piece: the segment that contains gbeg
    Piece cur = piece_at(gbeg);
    // a share may begin in the allowance behind a segment's last page: nothing to do there
    if (cur.pb >= cur.pe) cur = piece_next(cur, d, gbeg, gend);
    if (!cur.valid) return;

    uint32_t bad = 0;
    const int pf = partial_floats(g, D);
    float *ws_a = d.ws + (size_t)(2 * item) * pf;       // piece of a segment that began in an earlier share
    float *ws_b = ws_a + pf;                            // piece of a segment that begins in this share
    Pending pend_a, pend_b;
    pend_a.valid = pend_b.valid = 0;
    pend_a.arrived = pend_b.arrived = 0;

    // prologue of the stream: the first page pairs of the first piece, and its q
    constexpr int RING = Ring<D, DT, FLIGHT_KIB>::N;
    PairRegs<D, DT> ring[RING];
    PairIds pre;                            // block ids of the next pair to be requested
    RowInfo ri_c = row_info_uniform(d, cur.seq);       // the row of the piece being worked on
    {
        const int32_t *row = d.table + (size_t)ri_c.seq * d.row_stride;
        const int live_n = cur.n_pages > 0 ? cur.pe - cur.pb : 0;
#pragma unroll
        for (int r = 0; r < RING - 1; ++r)
            load_pair<D, DT>(ring[r], d, fetch_ids(d, row, cur.pb + 2 * r), 2 * r < live_n, 2 * r + 1 < live_n,
                             cur.kvh, lane, bad);
        pre = fetch_ids(d, row, cur.pb + 2 * (RING - 1));
    }
    bf16x8 qf[TL::NK], qn[TL::NK];
    load_q<D>(qf, d, ri_c, cur.kvh, lane, col);

    State<D, DT> st;
    // Instruction issue favours the older wave of a SIMD, and at two waves per SIMD the
    // younger one can starve for tens of microseconds before it gets its turn.  A wave
    // therefore starts at the highest priority and steps down as its share proceeds, so
    // whichever wave is behind is the one that is favoured.
    const uint32_t prio_total = gend - gbeg + 1;
    uint32_t prio_done = 0;
    int prio_lvl = 0;
    while (cur.valid) {
        const Piece nxt = piece_next(cur, d, gbeg, gend);
        const RowInfo ri_n = nxt.valid ? row_info_uniform(d, nxt.seq) : ri_c;
        // q of the next piece travels while this piece streams (of this piece again if there is no next)
        load_q<D>(qn, d, ri_n, nxt.valid ? nxt.kvh : cur.kvh, lane, col);
#pragma unroll
        for (int jt = 0; jt < TL::NV; ++jt) st.acc[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
        st.m = -INFINITY;
        st.l = 0.f;

        const int32_t *row_c = d.table + (size_t)ri_c.seq * d.row_stride;
        const int32_t *row_n = d.table + (size_t)ri_n.seq * d.row_stride;
        // whether this lane's column is a query of the row at all
        const bool col_live = n < g && col.tok < ri_c.ntok;
        const int n_live = cur.n_pages > 0 ? cur.pe - cur.pb : 0;       // pages to read and process
        const int n_next = (nxt.valid && nxt.n_pages > 0) ? nxt.pe - nxt.pb : 0;
        const int n_pairs = n_live > 0 ? (n_live + 1) >> 1 : 1;         // an empty segment still takes a turn
        const int last_valid = cur.L - (cur.n_pages - 1) * T;
        for (int t0 = 0; t0 < n_pairs; t0 += RING) {
            const bool last_turn = t0 + RING >= n_pairs;
#pragma unroll
            for (int r = 0; r < RING; ++r) {
                {
                    const int lvl = (int)(prio_done * 4u / prio_total) & 3;
                    if (lvl != prio_lvl) {
                        prio_lvl = lvl;
                        if (lvl == 1) __builtin_amdgcn_s_setprio(2);
                        else if (lvl == 2) __builtin_amdgcn_s_setprio(1);
                        else __builtin_amdgcn_s_setprio(0);
                    }
                }
                // request: position RING-1 of this turn (r == 0), else position r-1 of the next
                // turn, which belongs to the next piece when this is the piece's last turn
                {
                    const bool of_next = r > 0 && last_turn;
                    const int i = r == 0 ? 2 * (t0 + RING - 1) : (last_turn ? 2 * (r - 1) : 2 * (t0 + RING + r - 1));
                    const int lim = of_next ? n_next : n_live;
                    load_pair<D, DT>(ring[(r + RING - 1) % RING], d, pre, i < lim, i + 1 < lim,
                                     of_next ? nxt.kvh : cur.kvh, lane, bad);
                }
                // ids of the request after this one: the next step of this turn, or the first
                // step of the turn that follows (this piece's next turn, else the next piece's first)
                {
                    const int32_t *row;
                    int page;
                    if (r + 1 < RING) {
                        row = last_turn ? row_n : row_c;
                        page = last_turn ? nxt.pb + 2 * r : cur.pb + 2 * (t0 + RING + r);
                    } else {
                        row = last_turn ? row_n : row_c;
                        page = last_turn ? nxt.pb + 2 * (RING - 1) : cur.pb + 2 * (t0 + 2 * RING - 1);
                    }
                    pre = fetch_ids(d, row, page);
                }
                const int i = 2 * (t0 + r);
                if (i < n_live) {
                    const int pa = cur.pb + i;                                  // absolute page of the pair's first half
                    const int va = pa == cur.n_pages - 1 ? last_valid : T;
                    const int vb = i + 1 < n_live ? (pa + 1 == cur.n_pages - 1 ? last_valid : T) : 0;
                    process_pair<D, DT, false>(st, ring[r], qf, d.scale_log2, va, vb, G);
                    prio_done += 2;
                }
            }
        }

        // --- the piece is done: finish the segment or park a partial
        float *out_row = d.out + ((size_t)(ri_c.q0 + col.tok) * d.Hq + cur.kvh * d.g + col.head) * D;
        if (cur.n_pages == 0) {                  // empty context: the row is defined as zero
            if (cur.pb == 0 && col_live) {
#pragma unroll
                for (int jt = 0; jt < TL::NV; ++jt)
                    *reinterpret_cast<f32x4 *>(out_row + 16 * jt + 4 * G) = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        } else {
            float l = st.l;
            l += __shfl_xor(l, 16);
            l += __shfl_xor(l, 32);
            const uint32_t k0 = cut.index(cur.g0), k1 = cut.index(cur.g0 + (uint32_t)cur.n_pages - 1);
            if (k0 == k1) {                      // the whole segment was ours
                if (col_live) {
                    const float inv = 1.0f / l;
#pragma unroll
                    for (int jt = 0; jt < TL::NV; ++jt)
                        *reinterpret_cast<f32x4 *>(out_row + 16 * jt + 4 * G) = st.acc[jt] * inv;
                }
            } else {
                float *w = cur.pb == 0 ? ws_b : ws_a;
                if (col_live) {
#pragma unroll
                    for (int jt = 0; jt < TL::NV; ++jt)
                        *reinterpret_cast<f32x4 *>(w + n * D + 16 * jt + 4 * G) = st.acc[jt];
                    if (G == 0) {
                        w[g * D + n] = st.m;
                        w[g * D + g + n] = l;
                    }
                }
                // The partials and the arrival counters live in uncached device memory, so every
                // access goes to memory itself and is visible to all XCDs without flushing an L2.
                // Order is all that is left to enforce: the partial must have landed before the
                // counter moves.  The count itself is looked at only when the share is finished.
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                if (CACHED) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
                uint32_t arrived = 0;
                if (lane == 0) arrived = atomicAdd(d.cnt + (size_t)cur.seq * Hkv + cur.kvh, 1u);
                Pending &pd = cur.pb == 0 ? pend_b : pend_a;
                pd.valid = 1;
                pd.seq = cur.seq;
                pd.kvh = cur.kvh;
                pd.k0 = k0;
                pd.k1 = k1;
                pd.arrived = arrived;
            }
        }
        cur = nxt;
        ri_c = ri_n;
#pragma unroll
        for (int j = 0; j < TL::NK; ++j) qf[j] = qn[j];
    }

    // --- merges this wave owes: it arrived last at a segment shared with other waves
    if (w.stat && lane == 0) {          // tuning launches only: when did this XCD's waves finish streaming
        const unsigned xcd = blockIdx.x & 7u;
        atomicAdd(reinterpret_cast<unsigned long long *>(w.stat) + 2 * xcd, (unsigned long long)(wall_clock64() - t_begin));
        atomicAdd(reinterpret_cast<unsigned long long *>(w.stat) + 2 * xcd + 1, 1ull);
    }
    asm volatile("" ::: "memory");
    if (pend_a.valid) {
        const uint32_t arrived = (uint32_t)__builtin_amdgcn_readfirstlane((int)pend_a.arrived);
        if (arrived == pend_a.k1 - pend_a.k0) {
            // ready for the next launch (cached counters are cleared by the host before every launch instead)
            if (!CACHED && lane == 0) d.cnt[(size_t)pend_a.seq * Hkv + pend_a.kvh] = 0u;
            if (CACHED) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            merge_segment<D>(d, pend_a, lane, s_m, s_l);
        }
    }
    if (pend_b.valid) {
        const uint32_t arrived = (uint32_t)__builtin_amdgcn_readfirstlane((int)pend_b.arrived);
        if (arrived == pend_b.k1 - pend_b.k0) {
            if (!CACHED && lane == 0) d.cnt[(size_t)pend_b.seq * Hkv + pend_b.kvh] = 0u;
            if (CACHED) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            merge_segment<D>(d, pend_b, lane, s_m, s_l);
        }
    }
    if (bad && lane == 0) atomicOr(d.err, 1u);
}

__global__ __launch_bounds__(64, 2) void k_attention(const AttnGroup grp) {
    __shared__ float s_m[MAX_PIECES * 16], s_l[MAX_PIECES * 16];
    const int gi = blockIdx.x;
    int mi = 0;
    for (int i = 1; i < grp.n; ++i)
        if (gi >= grp.m[i].item_begin) mi = i;
    const AttnDesc &d = grp.m[mi];
    const int item = gi - d.item_begin;
    if (d.dtype == PKV_BF16) {
        if (d.D == 128) attn_wave<128, PKV_BF16>(d, grp.tune, item, s_m, s_l);
        else attn_wave<64, PKV_BF16>(d, grp.tune, item, s_m, s_l);
    } else {
        if (d.D == 128) attn_wave<128, PKV_E4M3>(d, grp.tune, item, s_m, s_l);
        else attn_wave<64, PKV_E4M3>(d, grp.tune, item, s_m, s_l);
    }
}

__global__ __launch_bounds__(64, 1) void k_attention_deep(const AttnGroup grp) {
    __shared__ float s_m[MAX_PIECES * 16], s_l[MAX_PIECES * 16];
    const int gi = blockIdx.x;
    int mi = 0;
    for (int i = 1; i < grp.n; ++i)
        if (gi >= grp.m[i].item_begin) mi = i;
    const AttnDesc &d = grp.m[mi];
    const int item = gi - d.item_begin;
    if (d.dtype == PKV_BF16) {
        if (d.D == 128) attn_wave<128, PKV_BF16, FLIGHT_KIB_1WAVE>(d, grp.tune, item, s_m, s_l);
        else attn_wave<64, PKV_BF16, FLIGHT_KIB_1WAVE>(d, grp.tune, item, s_m, s_l);
    } else {
        if (d.D == 128) attn_wave<128, PKV_E4M3, FLIGHT_KIB_1WAVE>(d, grp.tune, item, s_m, s_l);
        else attn_wave<64, PKV_E4M3, FLIGHT_KIB_1WAVE>(d, grp.tune, item, s_m, s_l);
    }
}

// The decode kernel for callers that may not allocate: the same code with its split-K partials and
// arrival counters in the library's file-scope scratch array (ordinary cached memory).
__global__ __launch_bounds__(64, 2) void k_attention_static(const AttnGroup grp) {
    __shared__ float s_m[MAX_PIECES * 16], s_l[MAX_PIECES * 16];
    const AttnDesc &d = grp.m[0];
    const int item = blockIdx.x;
    if (d.dtype == PKV_BF16) {
        if (d.D == 128) attn_wave<128, PKV_BF16, FLIGHT_KIB_2WAVES, true>(d, grp.tune, item, s_m, s_l);
        else attn_wave<64, PKV_BF16, FLIGHT_KIB_2WAVES, true>(d, grp.tune, item, s_m, s_l);
    } else {
        if (d.D == 128) attn_wave<128, PKV_E4M3, FLIGHT_KIB_2WAVES, true>(d, grp.tune, item, s_m, s_l);
        else attn_wave<64, PKV_E4M3, FLIGHT_KIB_2WAVES, true>(d, grp.tune, item, s_m, s_l);
    }
}

__global__ void k_clear_words(uint32_t *p, size_t n) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

// ---------------------------------------------------------------------------------
// Chunked prefill: causal attention of a group of consecutive query tokens against the
// paged cache (paper Sec. 5.2).  One work-group of four waves per (group, kv head).  Every
// wave owns two tiles of query tokens (a tile = 16 MFMA columns = tokens x the g heads of
// the kv head); the K and V tiles of a page pair are fetched once per work-group, one tile
// per wave, and passed through LDS in the very byte order they have in the block, so each
// wave reads its MFMA operands back with conflict-free LDS loads and uses each for both of
// its tiles.  Eight tiles share each byte fetched, against one in the decode kernel.
// `vmap` lists the groups like the rows of a decode launch, with up to 8 tiles of tokens
// each.  A group of few tokens in front of a long context may come as several work-groups,
// each with a part of the context; those leave partials that k_prefill_merge joins.
// NL x 1 KiB from the pool straight into LDS: lane l's 16 bytes at src + 1024 j land at
// dst + 1024 j + 16 l (the hardware adds the lane's offset to the LDS base held in M0).
// Written as assembly so that the compiler neither drains all loads in flight before the
// next one that targets the same LDS array, nor before LDS reads of another buffer; the
// waits are counted by hand where the data is needed (s_waitcnt vmcnt).
template <int NL>
__device__ __forceinline__ void lds_fill(const uint8_t *src, uint8_t *dst) {
    // wave-uniform by construction (the wave's tile of the buffer); tell the compiler so
    const uint32_t base = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(size_t)(__attribute__((address_space(3))) uint8_t *)dst);
    if (NL == 1)
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(base) : "memory", "m0");
    else if (NL == 2)
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off\n\tglobal_load_lds_dwordx4 %0, off offset:1024" ::"v"(src),
                     "s"(base)
                     : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off\n\tglobal_load_lds_dwordx4 %0, off offset:1024\n\t"
                     "global_load_lds_dwordx4 %0, off offset:2048\n\tglobal_load_lds_dwordx4 %0, off offset:3072" ::"v"(src),
                     "s"(base)
                     : "memory", "m0");
    static_assert(NL == 1 || NL == 2 || NL == 4, "tile sizes of 1, 2 or 4 KiB");
}

constexpr int PF_WAVES = 4;
constexpr int PF_TILES = 2;     // tiles of query tokens per wave: each operand read from LDS serves both
constexpr int PF_BUFS = 4;      // page pairs resident in LDS: one in use, three travelling
static_assert(PF_WAVES * PF_TILES == PKV_PREFILL_TILES, "host and kernel must agree on the group size");

template <int D, int DT>
__device__ __forceinline__ void prefill_group(const AttnDesc &d, uint8_t *lds0, uint8_t *lds1, uint8_t *lds2, uint8_t *lds3) {
    using TL = Tile<D, DT>;
    constexpr int NT = PF_TILES;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int G = lane >> 4, n = lane & 15;
    const int group = blockIdx.x / d.Hkv, kvh = blockIdx.x - group * d.Hkv;
    RowInfo gi = row_info_uniform(d, group);
    // a group of few query tokens in front of a long context comes as several work-groups, each with a
    // part of the context; they leave partial results that k_prefill_merge joins
    const int split = (gi.ntok >> 8) & 0xfff, n_split = gi.ntok >> 20;
    gi.ntok &= 0xff;
    const int tile_tok = d.cols / d.g;                      // query tokens per tile
    const Column col = column_of(d, n);
    // tokens the group's last query sees, never beyond what the row holds
    int L = PKV_CONST(int32_t, d.ctx_lens)[gi.seq] - gi.back;
    const int cap = PKV_CONST(int32_t, d.row_len)[gi.seq] * T;
    L = L < 0 ? 0 : (L > cap ? cap : L);
    L = __builtin_amdgcn_readfirstlane(L);
    const int n_pages = (L + T - 1) / T, n_pairs = (n_pages + 1) >> 1;
    const int last_valid = L - (n_pages - 1) * T;
    const int causal_from = L - (gi.ntok - 1);              // first token some column of the group may not see
    // the pairs this work-group walks
    const int per_split = n_split > 1 ? (n_pairs + n_split - 1) / n_split : n_pairs;
    const int p_begin = n_split > 1 ? (split * per_split < n_pairs ? split * per_split : n_pairs) : 0;
    const int p_end = p_begin + per_split < n_pairs ? p_begin + per_split : n_pairs;

    // this wave's tiles of the group: tile u covers the group's tokens [(w * NT + u) * tile_tok, ...)
    RowInfo ri[NT];
    bool col_live[NT];
    int col_lim[NT], tile_lim[NT];
    bf16x8 qf[NT][TL::NK];
    State<D, DT> st[NT];
#pragma unroll
    for (int u = 0; u < NT; ++u) {
        const int t0 = (w * NT + u) * tile_tok;
        ri[u].seq = gi.seq;
        ri[u].q0 = gi.q0 + t0;
        ri[u].back = 0;
        ri[u].ntok = gi.ntok - t0;
        ri[u].ntok = ri[u].ntok < 0 ? 0 : (ri[u].ntok > tile_tok ? tile_tok : ri[u].ntok);
        col_live[u] = n < d.cols && col.tok < ri[u].ntok;
        // the group's last token sees L; token i of the group sees L - (gi.ntok - 1 - i)
        col_lim[u] = col_live[u] ? L - (gi.ntok - 1 - (t0 + col.tok)) : L;
        tile_lim[u] = L - (gi.ntok - 1 - (t0 + ri[u].ntok - 1));      // what the tile's last token sees
        load_q<D>(qf[u], d, ri[u], kvh, lane, col);
#pragma unroll
        for (int jt = 0; jt < TL::NV; ++jt) st[u].acc[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
        st[u].m = -INFINITY;
        st[u].l = 0.f;
    }

    const int32_t *row = d.table + (size_t)gi.seq * d.row_stride;
    uint32_t bad = 0;

    // A pair travels from the pool straight into LDS (no staging registers), NBUF - 1 pairs ahead
    // of the one being worked on.  wave 0: K of page a, wave 1: V of page a, wave 2: K of page b,
    // wave 3: V of page b.  Every request issues exactly NL loads per lane (a page past the end is
    // replaced by the last one, and masked later), so the number of loads in flight tells which
    // pairs have landed.
    // The block id of a request is read through the scalar cache one request early (next_id), so
    // that the dependent chain table -> address -> load never waits inside a step.
    auto table_id = [&](int pair) {
        int page = 2 * pair + (w >> 1);
        page = page < n_pages ? page : n_pages - 1;
        page = page > 0 ? page : 0;
        const int last = d.row_stride - 1;
        // wave-uniform, and said to be: the id then comes through the scalar cache.  As a vector load
        // it would share the counter of the requests in flight, and waiting for it would drain them all.
        page = __builtin_amdgcn_readfirstlane(page < last ? page : last);
        return (uint32_t)PKV_CONST(int32_t, row)[page];
    };
    uint32_t next_id = table_id(p_begin);
    auto fetch = [&](int pair, uint8_t *buf) {
        uint32_t id = (uint32_t)__builtin_amdgcn_readfirstlane((int)next_id);
        next_id = table_id(pair + 1);
        const bool ok = id < d.max_block_id;
        if (!ok) {
            bad |= 1u;
            id = 0;
        }
        const uint32_t f = fastdiv_div(id, d.slots_div);
        const uint32_t sl = id - f * d.slots_div.d;
        const uint8_t *blk = d.pool_base + (uint64_t)f * d.frame_bytes + (uint64_t)sl * d.block_bytes +
                             (DT == PKV_E4M3 ? PKV_FP8_HEADER : 0);
        // an id outside the pool is never dereferenced: the same number of loads goes to a zeroed spare tile
        const uint8_t *src = (ok ? blk + ((size_t)kvh * 2 + (w & 1)) * TL::TILE_BYTES : reinterpret_cast<const uint8_t *>(d.safe)) + lane * 16;
        lds_fill<TL::NL>(src, buf + (size_t)w * TL::TILE_BYTES);
    };
    // wait until the loads of all but the `ahead` most recent requests have landed
    auto landed = [&](int ahead) {
        if (ahead >= 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * TL::NL) : "memory");
        else if (ahead == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(TL::NL) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    };
    // Operand registers of the pair being worked on.  The K tiles are read from LDS one step
    // ahead, right after the scores of the current pair have been issued (the registers are free
    // from then on), so that a step starts its matrix work without waiting for LDS; the V tiles
    // are read at the same point and arrive while the softmax arithmetic runs.
    PairRegs<D, DT> r;
    r.a.sk = r.a.sv = r.b.sk = r.b.sv = 1.f;
    // wave-uniform: does any token of pair p lie before what tile u sees
    auto sees = [&](int u, int p) { return ri[u].ntok > 0 && 2 * p * T < tile_lim[u]; };
    auto any_sees = [&](int p) {
        bool a = false;
#pragma unroll
        for (int u = 0; u < NT; ++u) a |= sees(u, p);
        return a && p < p_end;
    };
    auto read_k = [&](const uint8_t *buf) {
        const uint8_t *src = buf + lane * 16;
#pragma unroll
        for (int j = 0; j < TL::NL; ++j) {
            r.a.k[j] = *reinterpret_cast<const u32x4 *>(src + 0 * TL::TILE_BYTES + j * 1024);
            r.b.k[j] = *reinterpret_cast<const u32x4 *>(src + 2 * TL::TILE_BYTES + j * 1024);
        }
    };
    // bf16: the two pages' halves of an accumulation operand are read side by side into the four
    // registers of that operand (8-byte reads), so that no register moves are needed to join them
    u32x4 vop[DT == PKV_BF16 ? TL::NV : 1];
    // bf16: one LDS instruction per operand (ds_read2st64_b64: two 8-byte reads, 512-byte strides, into
    // four consecutive registers).  Left to itself the compiler fetches 16 bytes at a time and shuffles
    // the halves into place with 32 register moves per step.  The reads are issued here and waited for
    // in read_v_wait (the compiler does not count them; LDS returns in order, so its own waits stay safe).
    auto read_v = [&](const uint8_t *buf) {
        if constexpr (DT == PKV_BF16) {
            const uint32_t at = (uint32_t)(size_t)(__attribute__((address_space(3))) const uint8_t *)buf + (uint32_t)lane * 16u;
#pragma unroll
            for (int jt = 0; jt < TL::NV; ++jt) {
                constexpr int T512 = TL::TILE_BYTES / 512;
                const int o0 = T512 + 2 * (jt >> 1), o1 = 3 * T512 + 2 * (jt >> 1);
                const uint32_t a = at + (jt & 1) * 8u;
                asm volatile("ds_read2st64_b64 %0, %1 offset0:%2 offset1:%3" : "=v"(vop[jt]) : "v"(a), "n"(o0), "n"(o1) : "memory");
            }
        } else {
            const uint8_t *src = buf + lane * 16;
#pragma unroll
            for (int j = 0; j < TL::NL; ++j) {
                r.a.v[j] = *reinterpret_cast<const u32x4 *>(src + 1 * TL::TILE_BYTES + j * 1024);
                r.b.v[j] = *reinterpret_cast<const u32x4 *>(src + 3 * TL::TILE_BYTES + j * 1024);
            }
        }
    };
    auto read_v_wait = [&]() {
        if constexpr (DT == PKV_BF16) {
            static_assert(DT != PKV_BF16 || TL::NV == 8 || TL::NV == 4, "operand tiles of head dims 128 and 64");
            if constexpr (TL::NV == 8)
                asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(vop[0]), "+v"(vop[1]), "+v"(vop[2]), "+v"(vop[3]), "+v"(vop[TL::NV - 4]),
                             "+v"(vop[TL::NV - 3]), "+v"(vop[TL::NV - 2]), "+v"(vop[TL::NV - 1])::"memory");
            else
                asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(vop[0]), "+v"(vop[1]), "+v"(vop[2]), "+v"(vop[3])::"memory");
        }
    };
    // the per-page form of the V tiles that the masked path works on
    auto v_per_page = [&]() {
        if (DT == PKV_BF16) {
#pragma unroll
            for (int j = 0; j < TL::NL; ++j) {
                const u32x4 e = vop[DT == PKV_BF16 ? 2 * j : 0], o = vop[DT == PKV_BF16 ? 2 * j + 1 : 0];
                r.a.v[j] = mk4(e.x, e.y, o.x, o.y);
                r.b.v[j] = mk4(e.z, e.w, o.z, o.w);
            }
        }
    };
    // step p works on pair p (K already in registers, V in buf), reads the K tiles of pair p + 1
    // from buf_next, and sends the pair NBUF - 1 ahead into the buffer that pair p - 1 occupied
    auto step = [&](int p, const uint8_t *buf, const uint8_t *buf_next, uint8_t *refill) {
        const int pa = 2 * p;
        bool mine[NT];
        bool any_mine = false, all_mine = true;
#pragma unroll
        for (int u = 0; u < NT; ++u) {
            mine[u] = sees(u, p);
            any_mine |= mine[u];
            all_mine &= mine[u];
        }
        const bool next_mine = any_sees(p + 1);
        const int va = pa == n_pages - 1 ? last_valid : T;
        const int vb = pa + 1 < n_pages ? (pa + 1 == n_pages - 1 ? last_valid : T) : 0;
        const bool pair_tail = va < T || vb < T || (pa + 2) * T > causal_from;       // wave-uniform
        const bool fast = all_mine && !pair_tail;
        // The step's meeting point.  Before it, the wave's own requests for every pair up to p + 1 have
        // landed (the one for p + 2 may still travel); behind it, every wave's have, and every wave has
        // finished with pair p - 1: pair p + 1's K tiles may be read, and the buffer of pair p - 1 takes
        // the pair NBUF - 1 ahead.  A step needs neither for its score matrices (their K operands were
        // read a step ago), so on the common path the waves meet behind those: a wave that is ahead works
        // instead of waiting, and the requests, which would otherwise queue up behind each other where all
        // waves of a CU arrive together, are issued while the matrix instructions run.
        auto meet = [&]() {
            const int newest = p + PF_BUFS - 2 < p_end - 1 ? p + PF_BUFS - 2 : p_end - 1;
            landed(newest - (p + 1));
            __builtin_amdgcn_s_barrier();
        };
        if (!fast) meet();
        if (!fast && p + PF_BUFS - 1 < p_end) fetch(p + PF_BUFS - 1, refill);
        if (DT == PKV_E4M3 && any_mine) {
            const int last = d.row_stride - 1;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int page = pa + h;
                uint32_t id = (uint32_t)__builtin_amdgcn_readfirstlane(PKV_CONST(int32_t, row)[page < last ? page : last]);
                // past the end of the context, or an id outside the pool: no header is read
                const bool live = page < n_pages && id < d.max_block_id;
                if (!live) id = 0;
                const uint32_t f = fastdiv_div(id, d.slots_div);
                const uint32_t sl = id - f * d.slots_div.d;
                const float *hdr = live ? reinterpret_cast<const float *>(d.pool_base + (uint64_t)f * d.frame_bytes +
                                                                          (uint64_t)sl * d.block_bytes)
                                        : reinterpret_cast<const float *>(d.safe);
                float sk = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(PKV_CONST(float, hdr)[kvh])));
                float sv = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(PKV_CONST(float, hdr)[d.Hkv + kvh])));
                if (!live) sk = sv = 0.f;
                if (h == 0) { r.a.sk = sk; r.a.sv = sv; } else { r.b.sk = sk; r.b.sv = sv; }
            }
        }
        if (fast) {
            // the common case in one straight line: the score matrices of every tile, the operand
            // reads, the softmax of every tile, the accumulation of every tile
            f32x4 sa[NT], sb[NT];
            bf16x8 phv[NT], plv[NT];
            if constexpr (DT == PKV_BF16 && NT == 2) {
                pair_qk2<D>(r, qf[0], qf[1], sa, sb);
            } else {
#pragma unroll
                for (int u = 0; u < NT; ++u) pair_qk<D, DT>(r, qf[u], sa[u], sb[u]);
            }
            __builtin_amdgcn_sched_barrier(0);        // the K registers are rewritten below: not before their last use is issued
            meet();
            read_v(buf);
            if (next_mine) read_k(buf_next);
            if (p + PF_BUFS - 1 < p_end) fetch(p + PF_BUFS - 1, refill);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < NT; ++u) pair_softmax<D, DT>(st[u], r, sa[u], sb[u], d.scale_log2, phv[u], plv[u]);
            read_v_wait();
#pragma unroll
            for (int u = 0; u < NT; ++u) {
                if (DT == PKV_BF16) pair_accumulate_ops<D, DT>(st[u], vop, phv[u], plv[u]);
                else pair_accumulate<D, DT>(st[u], r, phv[u], plv[u]);
            }
        } else {
            if (any_mine) {
                read_v(buf);
                read_v_wait();
                v_per_page();
            }
#pragma unroll
            for (int u = 0; u < NT; ++u)
                if (mine[u]) {
                    if (pair_tail)
                        process_pair<D, DT, true, 2>(st[u], r, qf[u], d.scale_log2, va, vb, G, col_lim[u] - pa * T, true);
                    else
                        process_pair<D, DT, true, 1>(st[u], r, qf[u], d.scale_log2, va, vb, G);
                }
            __builtin_amdgcn_sched_barrier(0);
            if (next_mine) read_k(buf_next);
        }
    };

    // prologue: the first NBUF - 1 pairs are requested, the first two must have landed
    const int my_pairs = p_end - p_begin;
    if (my_pairs > 0) fetch(p_begin, lds0);
    if (my_pairs > 1) fetch(p_begin + 1, lds1);
    if (my_pairs > 2) fetch(p_begin + 2, lds2);
    landed((my_pairs < PF_BUFS - 1 ? my_pairs : PF_BUFS - 1) - 2);
    __builtin_amdgcn_s_barrier();
    // The queries were fetched with ordinary loads, which the compiler waits for where they are
    // first used.  That must not be inside the loop: the wait it would place there (it knows of
    // no other load) would drain the pair requests in flight in every step.  Use them here.
#pragma unroll
    for (int u = 0; u < NT; ++u)
#pragma unroll
        for (int j = 0; j < TL::NK; ++j) asm volatile("" ::"v"(qf[u][j]));
    if (any_sees(p_begin)) read_k(lds0);
    for (int p = p_begin; p < p_end; p += PF_BUFS) {
        step(p, lds0, lds1, lds3);
        if (p + 1 < p_end) step(p + 1, lds1, lds2, lds0);
        if (p + 2 < p_end) step(p + 2, lds2, lds3, lds1);
        if (p + 3 < p_end) step(p + 3, lds3, lds0, lds2);
    }

#pragma unroll
    for (int u = 0; u < NT; ++u) {
        float l = st[u].l;
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (n_split > 1) {
            // a part of the context: the unnormalised sums, the maximum and the denominator of every column
            float *part = d.ws + (((size_t)group * d.Hkv + kvh) * (PKV_PREFILL_TILES * 16) + (w * NT + u) * 16 + n) * (D + 4);
#pragma unroll
            for (int jt = 0; jt < TL::NV; ++jt) *reinterpret_cast<f32x4 *>(part + 16 * jt + 4 * G) = st[u].acc[jt];
            if (G == 0) {
                part[D] = st[u].m;
                part[D + 1] = l;
            }
        } else if (col_live[u]) {
            float *out_row = d.out + ((size_t)(ri[u].q0 + col.tok) * d.Hq + kvh * d.g + col.head) * D;
            const float inv = l > 0.f ? 1.0f / l : 0.f;          // no visible token: the row is defined as zero
#pragma unroll
            for (int jt = 0; jt < TL::NV; ++jt)
                *reinterpret_cast<f32x4 *>(out_row + 16 * jt + 4 * G) = st[u].acc[jt] * inv;
        }
    }
    if (bad && lane == 0) atomicOr(d.err, 1u);
}

// Joins the parts of a group whose context was walked by several work-groups of k_prefill: one
// work-group per (first part of such a group, kv head, tile of 16 columns); the parts are consecutive
// rows of d.vmap.  out = sum_i 2^(m_i - M) acc_i / sum_i 2^(m_i - M) l_i with M = max_i m_i, per column.
__global__ __launch_bounds__(256) void k_prefill_merge(const AttnDesc d) {
    const int tile = blockIdx.x % PKV_PREFILL_TILES, rk = blockIdx.x / PKV_PREFILL_TILES;
    const int row = rk / d.Hkv, kvh = rk - row * d.Hkv;
    const int4 e = d.vmap[row];
    const int split = (e.w >> 8) & 0xfff, n_split = e.w >> 20, ntok = e.w & 0xff;
    if (n_split <= 1 || split != 0) return;
    const int D = d.D, tile_tok = d.cols / d.g, stride = D + 4;       // D sums, the maximum, the denominator, two unused (16-byte rows)
    constexpr int NCOL = PKV_PREFILL_TILES * 16;
    const int quads = D / 4;
    for (int i = threadIdx.x; i < 16 * quads; i += blockDim.x) {
        const int n = i / quads, dq = i - n * quads;
        const int c = tile * 16 + n;
        const int tok = n / d.g, head = n - tok * d.g;
        const int t0 = tile * tile_tok;
        if (n >= d.cols || t0 + tok >= ntok) continue;            // a column without a query
        float M = -INFINITY;
        for (int s = 0; s < n_split; ++s) {
            const float *part = d.ws + (((size_t)(row + s) * d.Hkv + kvh) * NCOL + c) * stride;
            M = fmaxf(M, part[D]);
        }
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        float den = 0.f;
        for (int s = 0; s < n_split; ++s) {
            const float *part = d.ws + (((size_t)(row + s) * d.Hkv + kvh) * NCOL + c) * stride;
            const float m = part[D];
            const float f = m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m - M);
            den += f * part[D + 1];
            // a part that saw no token holds no usable sums (its factor is 0, its sums may be anything finite)
            if (f > 0.f) acc += *reinterpret_cast<const f32x4 *>(part + 4 * dq) * f;
        }
        const float inv = den > 0.f ? 1.0f / den : 0.f;
        float *out_row = d.out + ((size_t)(e.y + t0 + tok) * d.Hq + kvh * d.g + head) * D;
        *reinterpret_cast<f32x4 *>(out_row + 4 * dq) = acc * inv;
    }
}

__global__ __launch_bounds__(64 * PF_WAVES, 2) void k_prefill(const AttnDesc d) {
    // one array per buffer: distinct objects, so that a read of one buffer is not taken to depend
    // on the loads still travelling into the others; each holds a pair of the largest tiles (bf16, D = 128)
    __shared__ __align__(16) uint8_t lds0[4 * T * 128 * 2], lds1[4 * T * 128 * 2], lds2[4 * T * 128 * 2], lds3[4 * T * 128 * 2];
    if (d.dtype == PKV_BF16) {
        if (d.D == 128) prefill_group<128, PKV_BF16>(d, lds0, lds1, lds2, lds3);
        else prefill_group<64, PKV_BF16>(d, lds0, lds1, lds2, lds3);
    } else {
        if (d.D == 128) prefill_group<128, PKV_E4M3>(d, lds0, lds1, lds2, lds3);
        else prefill_group<64, PKV_E4M3>(d, lds0, lds1, lds2, lds3);
    }
}

// Read ceilings for comparison.  granule == 0: plain streaming read of the buffer,
// 16 bytes per lane.  granule > 0 (a power-of-two number of KiB): each wave reads
// whole granules of that size picked in a scrambled order, which is the access pattern
// of paged KV (contiguous inside a tile, scattered between tiles) without any math.
__global__ __launch_bounds__(256) void k_stream_read(const u32x4 *src, size_t n16, uint32_t granule16, uint32_t *sink) {
    u32x4 acc = {0, 0, 0, 0};
    if (granule16 == 0) {
        const size_t stride = (size_t)gridDim.x * blockDim.x;
        size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
        for (; i + 3 * stride < n16; i += 4 * stride) {
            const u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride);
            const u32x4 c = __builtin_nontemporal_load(src + i + 2 * stride),
                        e = __builtin_nontemporal_load(src + i + 3 * stride);
            acc ^= a ^ b ^ c ^ e;
        }
        for (; i < n16; i += stride) acc ^= __builtin_nontemporal_load(src + i);
    } else {
        const size_t n_gran = n16 / granule16;               // a power of two (checked by the host)
        const size_t waves = (size_t)gridDim.x * (blockDim.x / 64);
        const int lane = threadIdx.x & 63;
        for (size_t w = blockIdx.x * (size_t)(blockDim.x / 64) + (threadIdx.x >> 6); w < n_gran; w += waves) {
            const size_t gidx = (w * 0x9E3779B1ull + 12345ull) & (n_gran - 1);   // odd multiplier: a permutation
            const u32x4 *g = src + gidx * granule16 + lane;
            if (granule16 >= 8 * 64) {
                for (uint32_t k = 0; k < granule16; k += 8 * 64) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) acc ^= __builtin_nontemporal_load(g + k + u * 64);
                }
            } else {
                for (uint32_t k = 0; k < granule16; k += 64) acc ^= __builtin_nontemporal_load(g + k);
            }
        }
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) *sink = 1;   // keeps the loads alive
}

}  // namespace

hipError_t pkv_launch_attention(const AttnGroup &grp, bool deep, hipStream_t s, hipEvent_t *ev) {
    int items = 0;
    for (int i = 0; i < grp.n; ++i) items += grp.m[i].n_items;
    if (items == 0) return hipSuccess;
    hipError_t e;
    if (ev && (e = hipEventRecord(ev[0], s)) != hipSuccess) return e;
    if (deep) hipLaunchKernelGGL(k_attention_deep, dim3(items), dim3(64), 0, s, grp);
    else hipLaunchKernelGGL(k_attention, dim3(items), dim3(64), 0, s, grp);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (ev && (e = hipEventRecord(ev[1], s)) != hipSuccess) return e;
    return hipSuccess;
}

// ---- scratch of the entry point that allocates nothing ------------------------------------------
// Arrival counters first, split-K partials behind them.  Every GPU holds its own copy of the array
// at its own address; in host code the array's name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[PKV_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];     // per device: the address of its copy of `scratch`, once resolved
}  // namespace

// Address of the current device's copy of the scratch array (resolved once per device).
hipError_t pkv_static_scratch(void **ptr) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

// One model, the ordinary kernel form; d.ws and d.cnt point into the scratch array.  The counters the
// launch uses are cleared first (by a kernel: a caller may be capturing the stream into a graph).
hipError_t pkv_launch_attention_static(const AttnGroup &grp, uint32_t *cnt, size_t n_cnt, hipStream_t s) {
    if (grp.n != 1 || grp.m[0].n_items <= 0) return hipErrorInvalidValue;
    const unsigned blocks = (unsigned)((n_cnt + 255) / 256);
    hipLaunchKernelGGL(k_clear_words, dim3(blocks < 64 ? (blocks ? blocks : 1) : 64), dim3(256), 0, s, cnt, n_cnt);
    hipLaunchKernelGGL(k_attention_static, dim3(grp.m[0].n_items), dim3(64), 0, s, grp);
    return hipGetLastError();
}

hipError_t pkv_launch_prefill(const AttnDesc &d, int n_groups, bool any_split, hipStream_t s) {
    if (n_groups == 0) return hipSuccess;
    hipLaunchKernelGGL(k_prefill, dim3((unsigned)(n_groups * d.Hkv)), dim3(64 * PF_WAVES), 0, s, d);
    if (any_split)
        hipLaunchKernelGGL(k_prefill_merge, dim3((unsigned)(n_groups * d.Hkv * PKV_PREFILL_TILES)), dim3(256), 0, s, d);
    return hipGetLastError();
}

hipError_t pkv_launch_stream_read(const void *src, size_t bytes, size_t granule_bytes, uint32_t *sink, hipStream_t s) {
    hipLaunchKernelGGL(k_stream_read, dim3(256 * 16), dim3(256), 0, s, (const u32x4 *)src, bytes / 16,
                       (uint32_t)(granule_bytes / 16), sink);
    return hipGetLastError();
}
