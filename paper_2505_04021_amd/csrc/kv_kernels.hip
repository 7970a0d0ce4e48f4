// The write path of the shared pool (gfx950): bulk fill, the decode step's append of one
// new token per sequence, and a read-back in the logical layout.
//
// Paper: Sec. 4.2, D2 — a growing sequence takes its next token block from the slots of
// its model's pages; these kernels put K and V of the new tokens into that block, in the
// operand order the attention kernels read (kv_layout.h).
#include "kv_layout.h"

namespace {

// kv_write: logical [n_tok][Hkv][D] -> the in-block operand layouts.
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
    const int page = tok / PKV_T, t = tok % PKV_T;
    uint8_t *blk = block_ptr(d, (uint32_t)row[page]);
    if (DT == PKV_E4M3) {
        if (dd == 0) {
            const int srow = page - tok_begin / PKV_T;
            reinterpret_cast<float *>(blk)[h] = ks[(size_t)srow * Hkv + h];
            reinterpret_cast<float *>(blk)[Hkv + h] = vs[(size_t)srow * Hkv + h];
        }
        blk += PKV_FP8_HEADER;
    }
    const size_t tile = (size_t)PKV_T * D * E;
    uint8_t *kt = blk + (size_t)h * 2 * tile, *vt = kt + tile;
    if (DT == PKV_BF16) {
        reinterpret_cast<uint16_t *>(kt)[k_elem_off<DT>(t, dd)] = reinterpret_cast<const uint16_t *>(k)[idx];
        reinterpret_cast<uint16_t *>(vt)[v_elem_off<DT>(t, dd)] = reinterpret_cast<const uint16_t *>(v)[idx];
    } else {
        kt[k_elem_off<DT>(t, dd)] = k[idx];
        vt[v_elem_off<DT>(t, dd)] = v[idx];
    }
}

// kv_read: the inverse gather, plus the scale of each token's block.
template <int DT>
__global__ void k_kv_read(AttnDesc d, const int32_t *row, int tok_begin, int n_tok, uint8_t *k, uint8_t *v, float *ks,
                          float *vs) {
    constexpr int E = DT == PKV_BF16 ? 2 : 1;
    const int D = d.D, Hkv = d.Hkv;
    const int64_t total = (int64_t)n_tok * Hkv * D;
    const int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int dd = (int)(idx % D);
    const int h = (int)((idx / D) % Hkv);
    const int ti = (int)(idx / ((int64_t)D * Hkv));
    const int tok = tok_begin + ti;
    const int page = tok / PKV_T, t = tok % PKV_T;
    const uint8_t *blk = block_ptr(d, (uint32_t)row[page]);
    if (DT == PKV_E4M3) {
        if (dd == 0) {
            ks[(size_t)ti * Hkv + h] = reinterpret_cast<const float *>(blk)[h];
            vs[(size_t)ti * Hkv + h] = reinterpret_cast<const float *>(blk)[Hkv + h];
        }
        blk += PKV_FP8_HEADER;
    }
    const size_t tile = (size_t)PKV_T * D * E;
    const uint8_t *kt = blk + (size_t)h * 2 * tile, *vt = kt + tile;
    if (DT == PKV_BF16) {
        reinterpret_cast<uint16_t *>(k)[idx] = reinterpret_cast<const uint16_t *>(kt)[k_elem_off<DT>(t, dd)];
        reinterpret_cast<uint16_t *>(v)[idx] = reinterpret_cast<const uint16_t *>(vt)[v_elem_off<DT>(t, dd)];
    } else {
        k[idx] = kt[k_elem_off<DT>(t, dd)];
        v[idx] = vt[v_elem_off<DT>(t, dd)];
    }
}

// fp32 -> OCP E4M3 code: nearest value, ties to the even code, saturating at 448.
// Integer arithmetic on the bit pattern, so the result does not depend on a rounding
// mode or on how a conversion instruction treats the top of the range.
__device__ __forceinline__ uint32_t e4m3_encode(float y) {
    const uint32_t u = __float_as_uint(y);
    const uint32_t sign = (u >> 24) & 0x80u;
    const uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u) return 0x7fu;                    // NaN
    if (a >= 0x43e00000u) return sign | 0x7eu;            // |y| >= 448
    if (a < 0x3c800000u) {                                // |y| < 2^-6: subnormal codes, step 2^-9
        const float q = rintf(__uint_as_float(a) * 512.0f);   // exact scaling; ties to even
        return sign | (uint32_t)q;                        // 0 .. 8 (8 is the smallest normal)
    }
    uint32_t r = a + 0x7ffffu + ((a >> 20) & 1u);         // round to nearest even at mantissa bit 20
    r >>= 20;                                             // (biased exponent << 3) | 3 mantissa bits
    return sign | (r - ((127u - 7u) << 3));
}

__device__ __forceinline__ float e4m3_decode(uint32_t code) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const f32x2 p = __builtin_amdgcn_cvt_pk_f32_fp8((int)code, false);
    return p[0];
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}

// One K or V row of an e4m3 model: the running-maximum scale of its (block, kv head),
// re-encoding what the block already holds when the scale grows.  All arithmetic is
// fp32 with IEEE rounding (explicit _rn operations: nothing may be fused or reordered,
// the codes are compared bit for bit).
template <bool IS_V>
__device__ __forceinline__ void append_row_e4m3(uint8_t *tile, float *scale_p, int slot, int D, const uint16_t *x_bf16,
                                                int lane) {
    float x[2];
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int dd = lane + 64 * i;
        x[i] = dd < D ? bf16_bits_to_float(x_bf16[dd]) : 0.f;
        amax = fmaxf(amax, fabsf(x[i]));
    }
    amax = wave_max(amax);
    const float cand = __fdiv_rn(amax, 448.0f);
    float scale;
    if (slot == 0) {
        scale = amax > 0.f ? cand : 1.0f;
    } else {
        scale = *scale_p;
        if (cand > scale) {
            for (int t = 0; t < slot; ++t) {
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int dd = lane + 64 * i;
                    if (dd < D) {
                        uint8_t *c = tile + (IS_V ? v_elem_off<PKV_E4M3>(t, dd) : k_elem_off<PKV_E4M3>(t, dd));
                        const float v = __fmul_rn(e4m3_decode(*c), scale);
                        *c = (uint8_t)e4m3_encode(__fdiv_rn(v, cand));
                    }
                }
            }
            scale = cand;
        }
    }
    if (lane == 0) *scale_p = scale;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int dd = lane + 64 * i;
        if (dd < D)
            tile[IS_V ? v_elem_off<PKV_E4M3>(slot, dd) : k_elem_off<PKV_E4M3>(slot, dd)] =
                (uint8_t)e4m3_encode(__fdiv_rn(x[i], scale));
    }
}

// Several consecutive K or V rows of one page of an e4m3 model (slots slot0 .. slot0 + n - 1), with the
// same outcome, bit for bit, as append_row_e4m3 called for each in turn.  What those calls exchange
// through memory — the block's scale, the codes of the slots before — is held on chip here: the new rows
// and the codes the page already holds are fetched in one go, the rows are then taken in order (the scale
// rule is sequential by definition) with the page's codes in LDS, and codes and scale are written once.
// A lane only ever touches its own columns (lane and lane + 64), so the LDS arrays need no barrier.
template <bool IS_V>
__device__ __forceinline__ void append_rows_e4m3(uint8_t *tile, float *scale_p, int slot0, int n, int D, const uint16_t *x_bf16,
                                                 size_t row_stride, int lane, float (*sx)[128], uint8_t (*sc)[128]) {
    auto off = [&](int t, int dd) { return IS_V ? v_elem_off<PKV_E4M3>(t, dd) : k_elem_off<PKV_E4M3>(t, dd); };
    for (int t = 0; t < n; ++t)
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int dd = lane + 64 * i;
            if (dd < D) sx[slot0 + t][dd] = bf16_bits_to_float(x_bf16[(size_t)t * row_stride + dd]);
        }
    float scale = 1.0f;
    if (slot0 > 0) {
        scale = *scale_p;
        for (int t = 0; t < slot0; ++t)
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int dd = lane + 64 * i;
                if (dd < D) sc[t][dd] = tile[off(t, dd)];
            }
    }
    int first_changed = slot0;                       // slots below it still hold what memory holds
    for (int slot = slot0; slot < slot0 + n; ++slot) {
        float x[2];
        float amax = 0.f;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int dd = lane + 64 * i;
            x[i] = dd < D ? sx[slot][dd] : 0.f;
            amax = fmaxf(amax, fabsf(x[i]));
        }
        amax = wave_max(amax);
        const float cand = __fdiv_rn(amax, 448.0f);
        if (slot == 0) {
            scale = amax > 0.f ? cand : 1.0f;
        } else if (cand > scale) {
            for (int t = 0; t < slot; ++t)
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int dd = lane + 64 * i;
                    if (dd < D) {
                        const float v = __fmul_rn(e4m3_decode(sc[t][dd]), scale);
                        sc[t][dd] = (uint8_t)e4m3_encode(__fdiv_rn(v, cand));
                    }
                }
            scale = cand;
            first_changed = 0;
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int dd = lane + 64 * i;
            if (dd < D) sc[slot][dd] = (uint8_t)e4m3_encode(__fdiv_rn(x[i], scale));
        }
    }
    if (lane == 0) *scale_p = scale;
    for (int t = first_changed; t < slot0 + n; ++t)
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int dd = lane + 64 * i;
            if (dd < D) tile[off(t, dd)] = sc[t][dd];
        }
}

// kv_append: one wave per (sequence, kv head).  Without a chunk list it writes the token with
// index ctx_lens[seq] - 1 from row `seq` of k_new / v_new (bf16 [batch][Hkv][D]).  With one
// (d.vmap: per unit {first row of the sequence's new tokens, their number, sequence, which of the
// pages they touch}) it writes the sequence's new tokens at indices ctx_lens[seq] - tokens ..
// ctx_lens[seq] - 1 from consecutive rows, each exactly as a single append would (the e4m3 scale
// rule is sequential within a block by definition).
// A context length outside what the row holds is skipped and reported through the device
// error flags (bit 1).
template <int DT>
__global__ __launch_bounds__(64) void k_kv_append(AttnDesc d, const uint16_t *k_new, const uint16_t *v_new) {
    const int lane = threadIdx.x;
    const int unit = blockIdx.x / d.Hkv, h = blockIdx.x - unit * d.Hkv;
    const int D = d.D;
    // decode step: one wave per (sequence, kv head), one token.  Chunk: one wave per (sequence, kv
    // head, j-th page the chunk touches); where the chunk starts is known only here (ctx_lens is
    // device data), so the host lists one page more than the chunk can touch and a wave whose page
    // holds none of the chunk leaves.  Tokens of one page go in order (the e4m3 scale of a block
    // runs over its tokens); pages do not depend on each other (a block's scale starts afresh at
    // its first slot).
    int seq = unit, first_row = unit, n_new = 1, j = 0;
    if (d.vmap) {
        const int4 e = d.vmap[unit];
        first_row = e.x;
        n_new = e.y;
        seq = e.z;
        j = e.w;
        if (n_new == 0) return;
    }
    const int ctx = d.ctx_lens[seq];
    const int cap = d.row_len[seq] * PKV_T;
    if (ctx < n_new || ctx < 1 || ctx > cap) {
        if (lane == 0) atomicOr(d.err, 2u);
        return;
    }
    const int tok0 = ctx - n_new, page_j = tok0 / PKV_T + j;
    const int lo = tok0 > page_j * PKV_T ? tok0 : page_j * PKV_T;
    const int hi = ctx < (page_j + 1) * PKV_T ? ctx : (page_j + 1) * PKV_T;
    if (lo >= hi) return;
    const uint32_t id = (uint32_t)d.table[(size_t)seq * d.row_stride + page_j];
    if (id >= d.max_block_id) {
        if (lane == 0) atomicOr(d.err, 1u);
        return;
    }
    uint8_t *blk = block_ptr(d, id);
    if (DT == PKV_BF16) {
        // the elements of the page's new tokens do not depend on each other: all lanes, all tokens at once
        const size_t tile = (size_t)PKV_T * D * 2;
        uint16_t *kt = reinterpret_cast<uint16_t *>(blk + (size_t)h * 2 * tile);
        uint16_t *vt = reinterpret_cast<uint16_t *>(blk + (size_t)h * 2 * tile + tile);
        const size_t row0 = ((size_t)(first_row + (lo - tok0)) * d.Hkv + h) * D, stride = (size_t)d.Hkv * D;
        const int s0 = lo % PKV_T, n = hi - lo;
        if (n >= 4 && ((reinterpret_cast<uintptr_t>(k_new) | reinterpret_cast<uintptr_t>(v_new)) & 15) == 0) {
            // Several tokens of a chunk: whole 16-byte units.  A K unit is eight consecutive elements of
            // one token's row, as in the source; a V unit holds four consecutive tokens of one element
            // (8 bytes each for elements d and d + 16), gathered from four source rows.  Token groups the
            // chunk covers only in part go element by element.
            const int c8 = D >> 3;
            for (int e = lane; e < n * c8; e += 64) {
                const int t = e / c8, c = e - t * c8;
                *reinterpret_cast<uint4 *>(kt + k_elem_off<PKV_BF16>(s0 + t, 8 * c)) =
                    *reinterpret_cast<const uint4 *>(k_new + row0 + (size_t)t * stride + 8 * c);
            }
            for (int e = lane; e < 4 * D; e += 64) {
                const int G = e / D, dd = e - G * D;
                const int t_lo = 4 * G - s0;                       // the group's first token, counted from lo
                if (t_lo >= 0 && t_lo + 4 <= n) {
                    const uint16_t *src = v_new + row0 + (size_t)t_lo * stride + dd;
                    const uint32_t a = src[0], b = src[stride], c = src[2 * stride], f = src[3 * stride];
                    *reinterpret_cast<uint2 *>(vt + v_elem_off<PKV_BF16>(4 * G, dd)) = make_uint2(a | (b << 16), c | (f << 16));
                } else {
                    for (int k = 0; k < 4; ++k) {
                        const int t = t_lo + k;
                        if (t >= 0 && t < n) vt[v_elem_off<PKV_BF16>(4 * G + k, dd)] = v_new[row0 + (size_t)t * stride + dd];
                    }
                }
            }
            return;
        }
        const int n_el = n * D;
#pragma unroll 4
        for (int e = lane; e < n_el; e += 64) {
            const int t = e / D, dd = e - t * D;
            const size_t src = row0 + (size_t)t * stride + dd;
            kt[k_elem_off<PKV_BF16>(s0 + t, dd)] = k_new[src];
            vt[v_elem_off<PKV_BF16>(s0 + t, dd)] = v_new[src];
        }
        return;
    }
    if (hi - lo > 1) {
        // several tokens of a chunk in this page: in order, as single appends would, but in one pass
        __shared__ float sx[PKV_T][128];
        __shared__ uint8_t sc[PKV_T][128];
        float *hdr = reinterpret_cast<float *>(blk);
        const size_t tile = (size_t)PKV_T * D;
        uint8_t *kt = blk + PKV_FP8_HEADER + (size_t)h * 2 * tile, *vt = kt + tile;
        const size_t src = ((size_t)(first_row + (lo - tok0)) * d.Hkv + h) * D, stride = (size_t)d.Hkv * D;
        append_rows_e4m3<false>(kt, hdr + h, lo % PKV_T, hi - lo, D, k_new + src, stride, lane, sx, sc);
        append_rows_e4m3<true>(vt, hdr + d.Hkv + h, lo % PKV_T, hi - lo, D, v_new + src, stride, lane, sx, sc);
        return;
    }
    for (int tok = lo; tok < hi; ++tok) {
        const int i = tok - tok0, slot = tok % PKV_T;
        const uint16_t *kx = k_new + ((size_t)(first_row + i) * d.Hkv + h) * D;
        const uint16_t *vx = v_new + ((size_t)(first_row + i) * d.Hkv + h) * D;
        {
            float *hdr = reinterpret_cast<float *>(blk);
            const size_t tile = (size_t)PKV_T * D;
            uint8_t *kt = blk + PKV_FP8_HEADER + (size_t)h * 2 * tile, *vt = kt + tile;
            append_row_e4m3<false>(kt, hdr + h, slot, D, kx, lane);
            append_row_e4m3<true>(vt, hdr + d.Hkv + h, slot, D, vx, lane);
            // the next token of the chunk may read this block's codes and scale (written by other lanes)
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
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

hipError_t pkv_launch_kv_read(const AttnDesc &d, int seq, int tok_begin, int n_tok, void *k, void *v, float *ks, float *vs,
                              hipStream_t s) {
    const int64_t total = (int64_t)n_tok * d.Hkv * d.D;
    if (total == 0) return hipSuccess;
    const int32_t *row = d.table + (size_t)seq * d.row_stride;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (d.dtype == PKV_BF16)
        hipLaunchKernelGGL(k_kv_read<PKV_BF16>, dim3(blocks), dim3(256), 0, s, d, row, tok_begin, n_tok, (uint8_t *)k,
                           (uint8_t *)v, ks, vs);
    else
        hipLaunchKernelGGL(k_kv_read<PKV_E4M3>, dim3(blocks), dim3(256), 0, s, d, row, tok_begin, n_tok, (uint8_t *)k,
                           (uint8_t *)v, ks, vs);
    return hipGetLastError();
}

hipError_t pkv_launch_kv_append(const AttnDesc &d, const void *k_new, const void *v_new, hipStream_t s) {
    if (d.batch == 0) return hipSuccess;
    const unsigned blocks = (unsigned)(d.batch * d.Hkv);
    if (d.dtype == PKV_BF16)
        hipLaunchKernelGGL(k_kv_append<PKV_BF16>, dim3(blocks), dim3(64), 0, s, d, (const uint16_t *)k_new,
                           (const uint16_t *)v_new);
    else
        hipLaunchKernelGGL(k_kv_append<PKV_E4M3>, dim3(blocks), dim3(64), 0, s, d, (const uint16_t *)k_new,
                           (const uint16_t *)v_new);
    return hipGetLastError();
}
