// Matrix-core kernels for the dense cases: shared negatives and the full catalogue, bf16 inputs.
//
// With one list of negatives for the whole batch the indexed scalar products of Alg. 1 / Alg. 2 become the dense
// contraction H x E_neg^T; in full-catalogue mode (Sec. 3.1, Eq. 2) E_neg is the whole table.  One kernel template
// serves the three passes.  A "stationary" operand X lives in registers, one row per lane column, and a "streamed"
// operand Y goes through LDS in tiles shared by the four wavefronts of a workgroup:
//
//   FWD : X = hidden states,  Y = candidate rows.  S^T = Y X^T on the matrix cores, online max / sum-exp per lane (Alg. 1).
//   DH  : X = hidden states,  Y = candidate rows.  P^T = exp(S^T - LSE), dH^T += Y^T P^T          (Alg. 2, Eq. 6 left).
//   DE  : X = candidate rows, Y = hidden states.   G   = g exp(S - LSE),  dE_neg^T += Y^T G       (Alg. 2, Eq. 6 right).
//
// Scores are produced transposed (streamed index in the accumulator registers, stationary index on the lanes) so that
// the softmax reduction of FWD needs no cross-lane traffic until the very end, and so that the probability tile can be
// fed back as the B operand of the second product straight from registers: the permutation the accumulator layout
// imposes on the reduction index is matched by reading the A operand with the LDS transpose loads of gfx950.
//
// The correct item is not a column of the dense tile.  Its score is taken separately (the paper's correct-logit
// kernel) and enters with a per-position weight w_i = 1 - c_i, c_i = number of negatives equal to the position's own
// target: the dense tile counts those c_i copies, the definition wants the target exactly once, so
//   sum_live exp(o) = sum_k exp(o_ik) + w_i exp(o+_i),   coefficient of the correct item = g_i (w_i p+_i - 1).
// With collision masking off w_i = 1; in full-catalogue mode the target is already one of the columns and w_i = 0.
#include "cce_device.hpp"
#include "cce_kernels.hpp"

namespace cce {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int kThreads = 256;
constexpr int kXPerWave = 32;
constexpr int kXPerBlock = 128;
constexpr int kPad = 8;  // bf16 elements of padding per LDS row

enum { MODE_FWD = 0, MODE_DH = 1, MODE_DE = 2 };

__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    f32x2 v = {lo, hi};
    bf16x2 b = __builtin_convertvector(v, bf16x2);  // round to nearest even
    uint32_t u;
    __builtin_memcpy(&u, &b, 4);
    return u;
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v)
{
    bf16x8 r;
    __builtin_memcpy(&r, &v, 16);
    return r;
}

// Position row of compacted index x (identity when there is no mask).
__device__ __forceinline__ int64_t pos_row(const TileArgs &a, int64_t x) { return a.idx ? (int64_t)a.idx[x] : x; }
// Item row of candidate column k (identity in full-catalogue mode).
__device__ __forceinline__ int64_t item_row(const TileArgs &a, int64_t k)
{
    if (!a.neg) return k;
    int64_t id = a.neg[k];
    if (a.validate && (id < 0 || id >= a.V)) id = 0;  // flagged by the preparation kernel; never dereferenced
    return id;
}

// Dot product of the lane's half of a stationary row (chunks kk*16 + hi*8 .. +8) with the same chunks of another row.
template <int D>
__device__ __forceinline__ float half_row_dot(const uint4 (&xr)[D / 16], const uint16_t *other, int hi)
{
    float s = 0.f;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
        const uint4 o = *reinterpret_cast<const uint4 *>(other + kk * 16 + hi * 8);
        s = fmaf(bf16_lo(xr[kk].x), bf16_lo(o.x), s);
        s = fmaf(bf16_hi(xr[kk].x), bf16_hi(o.x), s);
        s = fmaf(bf16_lo(xr[kk].y), bf16_lo(o.y), s);
        s = fmaf(bf16_hi(xr[kk].y), bf16_hi(o.y), s);
        s = fmaf(bf16_lo(xr[kk].z), bf16_lo(o.z), s);
        s = fmaf(bf16_hi(xr[kk].z), bf16_hi(o.z), s);
        s = fmaf(bf16_lo(xr[kk].w), bf16_lo(o.w), s);
        s = fmaf(bf16_hi(xr[kk].w), bf16_hi(o.w), s);
    }
    return s;
}

template <int D, int MODE, int BY>
__global__ __launch_bounds__(kThreads, 2) void tile_kernel(TileArgs a)
{
    constexpr int KK = D / 16;           // k-steps of the score product
    constexpr int MB = D / 32;           // 32-row output blocks of the second product
    constexpr int ROW = D + kPad;        // LDS row pitch in elements
    constexpr int CPR = D / 8;           // 16-byte chunks per row
    constexpr int CH = BY * CPR / kThreads;  // chunks staged per thread and tile
    static_assert(BY * CPR % kThreads == 0, "tile must split evenly over the threads");

    __shared__ __attribute__((aligned(16))) uint16_t ytile[2][BY * ROW];
    __shared__ float yconst[2][BY];
    __shared__ uint32_t ysign[2][BY];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int lo = lane & 31;
    const int hi = lane >> 5;

    const int64_t n_pos = a.n_valid_ptr ? (int64_t)*a.n_valid_ptr : a.N;
    const int64_t n_x = (MODE == MODE_DE) ? a.n_cols : n_pos;
    const int64_t n_y = (MODE == MODE_DE) ? n_pos : a.n_cols;
    const int split = blockIdx.x % a.splits;
    const int64_t xb = blockIdx.x / a.splits;
    if (xb * kXPerBlock >= n_x) return;  // whole block past the end (the grid is sized for the unmasked N)

    const uint16_t *Xbase = (MODE == MODE_DE) ? a.E : a.H;
    const uint16_t *Ybase = (MODE == MODE_DE) ? a.H : a.E;

    // ---- stationary rows -> registers in B-operand layout: lane (lo, hi) holds X[x][kk*16 + hi*8 .. +8]
    const int64_t x = xb * kXPerBlock + wave * kXPerWave + lo;
    const bool x_ok = x < n_x;
    const int64_t xrow = (MODE == MODE_DE) ? item_row(a, x_ok ? x : 0) : pos_row(a, x_ok ? x : 0);
    uint4 xr[KK];
    {
        const uint16_t *xp = Xbase + xrow * D;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) xr[kk] = *reinterpret_cast<const uint4 *>(xp + kk * 16 + hi * 8);
    }
    float cx = 0.f;  // DH: -lse * log2(e) of the lane's position
    if (MODE == MODE_DH) cx = -a.lse_in[xrow] * kLog2e;

    // ---- range of streamed tiles of this split
    const int64_t n_tiles = (n_y + BY - 1) / BY;
    const int64_t t_begin = n_tiles * split / a.splits;
    const int64_t t_end = n_tiles * (split + 1) / a.splits;

    f32x16 acc[MODE == MODE_FWD ? 1 : MB];
    if (MODE != MODE_FWD) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[mb][q] = 0.f;
    }
    float run_m = -INFINITY, run_s = 0.f;  // FWD: base-2 running max and sum of this lane's half of the candidates

    uint4 stage[CH];
    float stage_c = 0.f;
    uint32_t stage_s = 0;
    auto load_tile = [&](int64_t t) {
        const int64_t y0 = t * BY;
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int c = tid + u * kThreads;
            const int r = c / CPR, col = c % CPR;
            const int64_t y = y0 + r;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (y < n_y) {
                const int64_t row = (MODE == MODE_DE) ? pos_row(a, y) : item_row(a, y);
                v = *reinterpret_cast<const uint4 *>(Ybase + row * D + col * 8);
            }
            stage[u] = v;
        }
        if (MODE == MODE_DE && tid < BY) {
            const int64_t y = y0 + tid;
            stage_c = -INFINITY;
            stage_s = 0;
            if (y < n_y) {
                const int64_t row = pos_row(a, y);
                const float g = a.g ? a.g[row] : 1.f;
                // g * exp(o - lse) = sign(g) * 2^(o log2e - lse log2e + log2|g|)
                stage_c = -a.lse_in[row] * kLog2e + __builtin_amdgcn_logf(fabsf(g));
                stage_s = __float_as_uint(g) & 0x80000000u;
            }
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int c = tid + u * kThreads;
            const int r = c / CPR, col = c % CPR;
            *reinterpret_cast<uint4 *>(&ytile[buf][r * ROW + col * 8]) = stage[u];
        }
        if (MODE == MODE_DE && tid < BY) {
            yconst[buf][tid] = stage_c;
            ysign[buf][tid] = stage_s;
        }
    };

    if (t_begin < t_end) {
        load_tile(t_begin);
        store_tile(0);
    }
    __syncthreads();

    for (int64_t t = t_begin; t < t_end; ++t) {
        const int buf = (int)((t - t_begin) & 1);
        if (t + 1 < t_end) load_tile(t + 1);

#pragma unroll
        for (int sb = 0; sb < BY / 32; ++sb) {
            // ---- S^T tile: rows = 32 streamed y, columns = the wavefront's 32 stationary x
            f32x16 s;
#pragma unroll
            for (int q = 0; q < 16; ++q) s[q] = 0.f;
            const uint16_t *arow = &ytile[buf][(sb * 32 + lo) * ROW + hi * 8];
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const uint4 av = *reinterpret_cast<const uint4 *>(arow + kk * 16);
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(av), as_bf16x8(xr[kk]), s, 0, 0, 0);
            }
            // accumulator register q of lane (lo, hi) holds y = sb*32 + (q/4)*8 + hi*4 + q%4

            if (MODE == MODE_FWD) {
                const int64_t ybase = t * BY + sb * 32 + hi * 4;
                if (t * BY + sb * 32 + 32 > n_y) {  // ragged last tile: rows past the end do not take part
#pragma unroll
                    for (int q = 0; q < 16; ++q)
                        if (ybase + (q / 4) * 8 + (q % 4) >= n_y) s[q] = -INFINITY;
                }
                float tm = s[0];
#pragma unroll
                for (int q = 1; q < 16; ++q) tm = fmaxf(tm, s[q]);
                const float mn = fmaxf(run_m, tm * kLog2e);
                if (mn > -INFINITY) {
                    float part = 0.f;
#pragma unroll
                    for (int q = 0; q < 16; ++q) part += __builtin_amdgcn_exp2f(fmaf(s[q], kLog2e, -mn));
                    run_s = run_s * __builtin_amdgcn_exp2f(run_m - mn) + part;
                    run_m = mn;
                }
            } else {
                // ---- probabilities (DH) or coefficients (DE), rounded to bf16, as the B operand of the second product
                uint32_t gp[8];
                if (MODE == MODE_DH) {
#pragma unroll
                    for (int q = 0; q < 16; q += 2)
                        gp[q / 2] = pack2(__builtin_amdgcn_exp2f(fmaf(s[q], kLog2e, cx)),
                                          __builtin_amdgcn_exp2f(fmaf(s[q + 1], kLog2e, cx)));
                } else {
#pragma unroll
                    for (int qq = 0; qq < 4; ++qq) {
                        const float4 cy = *reinterpret_cast<const float4 *>(&yconst[buf][sb * 32 + qq * 8 + hi * 4]);
                        const uint4 sg = *reinterpret_cast<const uint4 *>(&ysign[buf][sb * 32 + qq * 8 + hi * 4]);
                        const float g0 = __uint_as_float(__float_as_uint(__builtin_amdgcn_exp2f(fmaf(s[qq * 4 + 0], kLog2e, cy.x))) | sg.x);
                        const float g1 = __uint_as_float(__float_as_uint(__builtin_amdgcn_exp2f(fmaf(s[qq * 4 + 1], kLog2e, cy.y))) | sg.y);
                        const float g2 = __uint_as_float(__float_as_uint(__builtin_amdgcn_exp2f(fmaf(s[qq * 4 + 2], kLog2e, cy.z))) | sg.z);
                        const float g3 = __uint_as_float(__float_as_uint(__builtin_amdgcn_exp2f(fmaf(s[qq * 4 + 3], kLog2e, cy.w))) | sg.w);
                        gp[qq * 2 + 0] = pack2(g0, g1);
                        gp[qq * 2 + 1] = pack2(g2, g3);
                    }
                }
                // ---- out^T[t, x] += sum_y Y[y, t] * G^T[y, x]; the A operand is read transposed from the row-major tile
                const int j = lane & 15, ta = j >> 2, tb = j & 3, cb = (lane >> 4) & 1;
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2) {
                    const uint4 bv = make_uint4(gp[k2 * 4 + 0], gp[k2 * 4 + 1], gp[k2 * 4 + 2], gp[k2 * 4 + 3]);
                    const uint16_t *tbase = &ytile[buf][(sb * 32 + k2 * 16 + hi * 4 + ta) * ROW + cb * 16 + tb * 4];
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        typedef s16x4 __attribute__((address_space(3))) * lds_v4;
                        const s16x4 r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(tbase + mb * 32));
                        const s16x4 r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(tbase + mb * 32 + 8 * ROW));
                        const s16x8 r = __builtin_shufflevector(r0, r1, 0, 1, 2, 3, 4, 5, 6, 7);
                        bf16x8 av;
                        __builtin_memcpy(&av, &r, 16);
                        acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, as_bf16x8(bv), acc[mb], 0, 0, 0);
                    }
                }
            }
        }

        if (t + 1 < t_end) store_tile(buf ^ 1);
        __syncthreads();
    }

    // =====================================================================================================  epilogues
    if (MODE == MODE_FWD) {
        // merge the two halves of the candidates that lanes (lo,0) and (lo,1) hold for the same position
        {
            const float m2 = __shfl_xor(run_m, 32, 64), s2 = __shfl_xor(run_s, 32, 64);
            const float M = fmaxf(run_m, m2);
            if (M > -INFINITY) {
                run_s = run_s * __builtin_amdgcn_exp2f(run_m - M) + s2 * __builtin_amdgcn_exp2f(m2 - M);
                run_m = M;
            }
        }
        if (a.splits > 1) {
            if (x_ok && hi == 0) {
                a.part_m[(int64_t)split * a.N + x] = run_m;
                a.part_s[(int64_t)split * a.N + x] = run_s;
            }
            return;
        }
        float op = 0.f;
        if (x_ok) op = half_row_dot<D>(xr, a.E + (int64_t)a.tgt[xrow] * D, hi);
        op += __shfl_xor(op, 32, 64);
        if (x_ok && hi == 0) {
            const float w = a.pos_weight_mode == 2 ? 0.f : (a.cnt ? 1.f - (float)a.cnt[xrow] : 1.f);
            const float o2 = op * kLog2e;
            const float M = (w != 0.f) ? fmaxf(run_m, o2) : run_m;
            const float tot = run_s * __builtin_amdgcn_exp2f(run_m - M) + w * __builtin_amdgcn_exp2f(o2 - M);
            const float l = (M + __builtin_amdgcn_logf(tot)) * kLn2;
            a.lse[xrow] = l;
            a.loss[xrow] = l - op;
        }
    } else if (MODE == MODE_DH) {
        if (a.splits > 1) {
            if (x_ok) {
                float *dst = a.part_dH + ((int64_t)split * a.N + x) * D;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int qq = 0; qq < 4; ++qq)
                        *reinterpret_cast<float4 *>(dst + mb * 32 + qq * 8 + hi * 4) =
                            make_float4(acc[mb][qq * 4], acc[mb][qq * 4 + 1], acc[mb][qq * 4 + 2], acc[mb][qq * 4 + 3]);
            }
            return;
        }
        float op = 0.f;
        const uint16_t *erow = a.E + (x_ok ? (int64_t)a.tgt[xrow] : 0) * D;
        if (x_ok) op = half_row_dot<D>(xr, erow, hi);
        op += __shfl_xor(op, 32, 64);
        if (x_ok) {
            const float w = a.pos_weight_mode == 2 ? 0.f : (a.cnt ? 1.f - (float)a.cnt[xrow] : 1.f);
            const float pp = __builtin_amdgcn_exp2f(fmaf(op, kLog2e, cx));
            const float cpos = w * pp - 1.f;  // coefficient of the correct item before the upstream gradient
            const float g = a.g ? a.g[xrow] : 1.f;
            if (hi == 0) a.coef[xrow] = g * cpos;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int qq = 0; qq < 4; ++qq) {
                    const int col = mb * 32 + qq * 8 + hi * 4;
                    const uint2 ev = *reinterpret_cast<const uint2 *>(erow + col);
                    const float v0 = g * fmaf(cpos, bf16_lo(ev.x), acc[mb][qq * 4 + 0]);
                    const float v1 = g * fmaf(cpos, bf16_hi(ev.x), acc[mb][qq * 4 + 1]);
                    const float v2 = g * fmaf(cpos, bf16_lo(ev.y), acc[mb][qq * 4 + 2]);
                    const float v3 = g * fmaf(cpos, bf16_hi(ev.y), acc[mb][qq * 4 + 3]);
                    if (a.dH_bf16) {
                        *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(a.dH) + xrow * D + col) =
                            make_uint2(pack2(v0, v1), pack2(v2, v3));
                    } else {
                        *reinterpret_cast<float4 *>(static_cast<float *>(a.dH) + xrow * D + col) = make_float4(v0, v1, v2, v3);
                    }
                }
        }
    } else {
        // dE_neg^T sits in the accumulators with the hidden index in registers and the candidate row on the lanes.
        // Turn each 32x32 block round through LDS (the streamed tiles are dead by now) so that one atomic
        // instruction adds 32 consecutive floats to each of two table rows.
        float *tbuf = reinterpret_cast<float *>(&ytile[0][0]) + wave * (32 * 33);
        static_assert(sizeof(ytile) >= 4 * 32 * 33 * sizeof(float), "staging tiles too small for the dE transpose");
        __shared__ int64_t xrow_s[kXPerBlock];
        xrow_s[wave * kXPerWave + lo] = x_ok ? xrow : -1;  // both half-waves write the same value
        __syncthreads();
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
            for (int q = 0; q < 16; ++q) tbuf[lo * 33 + (q / 4) * 8 + hi * 4 + (q % 4)] = acc[mb][q];
            __syncthreads();
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int xr_local = r * 2 + hi;
                const int64_t row = xrow_s[wave * kXPerWave + xr_local];
                const float v = tbuf[xr_local * 33 + lo];
                if (row >= 0) unsafeAtomicAdd(a.dE + row * D + mb * 32 + lo, v);
            }
            __syncthreads();
        }
    }
}

// ---------------------------------------------------------------------------------------------------------------------
// Preparation: compaction of the valid positions, zero rows for the padded ones, and the multiplicity c_i of each
// position's target among the shared negatives (through a hash table of the negatives built in LDS by every block).
constexpr int kPrepThreads = 1024;
constexpr int kTgtSlots = 2048;  // LDS hash table of the block's own targets; load factor <= 1/2, so probing always ends

__device__ __forceinline__ uint32_t hash_id(int32_t id, int slots) { return (((uint32_t)id * 2654435761u) >> 15) & (uint32_t)(slots - 1); }

// Number of non-zero bytes in a 32-bit word.
__device__ __forceinline__ int nonzero_bytes(uint32_t w)
{
    return __popc((w | ((w & 0x7f7f7f7fu) + 0x7f7f7f7fu)) & 0x80808080u);
}

// Every block handles 1024 consecutive positions.  The slot of a valid position in the compacted list is its rank
// among all valid positions, so the list keeps the original order and needs no atomics: a block finds the number of
// valid positions in front of it by counting the mask bytes of that prefix itself (N bytes at most, from L2).
__global__ __launch_bounds__(kPrepThreads) void prep_kernel(PrepArgs p)
{
    __shared__ int32_t hkey[kTgtSlots];
    __shared__ int32_t hcnt[kTgtSlots];
    __shared__ int32_t wave_count[kPrepThreads / 64];
    __shared__ int32_t wave_prefix[kPrepThreads / 64];
    __shared__ int32_t block_base;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t i0 = (int64_t)blockIdx.x * kPrepThreads;
    const int64_t i = i0 + tid;
    bool valid = false;
    int32_t ti = 0;
    if (i < p.N) {
        valid = (p.mask == nullptr) || (p.mask[i] != 0);
        if (valid) {
            ti = p.tgt[i];
            if (p.validate && (ti < 0 || (int64_t)ti >= p.V)) {
                valid = false;
                atomicOr(p.header + kHdrStatus, 1);
            }
        }
    }

    if (p.idx) {
        // ---- valid positions in front of this block
        int32_t before = 0;
        if (p.validate) {  // validity depends on the target too: walk positions one by one
            for (int64_t j = tid; j < i0; j += kPrepThreads) {
                const bool m = (p.mask == nullptr) || (p.mask[j] != 0);
                if (m) {
                    const int32_t t = p.tgt[j];
                    before += (t >= 0 && (int64_t)t < p.V) ? 1 : 0;
                }
            }
        } else if (p.mask) {  // i0 is a multiple of 1024, the mask is 16-byte aligned
            const uint4 *m16 = reinterpret_cast<const uint4 *>(p.mask);
            for (int64_t c = tid; c < i0 / 16; c += kPrepThreads) {
                const uint4 v = m16[c];
                before += nonzero_bytes(v.x) + nonzero_bytes(v.y) + nonzero_bytes(v.z) + nonzero_bytes(v.w);
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) before += __shfl_xor(before, off, 64);
        const uint64_t ballot = __ballot(valid);
        const int rank_in_wave = __popcll(ballot & ((1ull << lane) - 1ull));
        if (lane == 0) {
            wave_count[wave] = __popcll(ballot);
            wave_prefix[wave] = before;  // partial sum of the prefix count held by this wavefront
        }
        __syncthreads();
        if (tid == 0) {
            int32_t base = 0, run = 0;
            for (int w = 0; w < kPrepThreads / 64; ++w) base += wave_prefix[w];
            for (int w = 0; w < kPrepThreads / 64; ++w) {
                const int32_t c = wave_count[w];
                wave_count[w] = run;
                run += c;
            }
            block_base = base;
            if (blockIdx.x == gridDim.x - 1) p.header[kHdrNValid] = base + run;  // the last block knows the total
        }
        __syncthreads();
        if (valid) p.idx[block_base + wave_count[wave] + rank_in_wave] = (int32_t)i;
    }

    // ---- rows of padded positions are zero
    if (i < p.N && !valid) {
        if (p.loss) p.loss[i] = 0.f;
        if (p.lse) p.lse[i] = 0.f;
        if (p.dH) {
            if (p.dH_bf16) {
                uint4 *row = reinterpret_cast<uint4 *>(static_cast<uint16_t *>(p.dH) + i * p.d);
                for (int c = 0; c < p.d / 8; ++c) row[c] = make_uint4(0, 0, 0, 0);
            } else {
                float4 *row = reinterpret_cast<float4 *>(static_cast<float *>(p.dH) + i * p.d);
                for (int c = 0; c < p.d / 4; ++c) row[c] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    }

    // ---- multiplicity of each target among the shared negatives: the block's targets go into an LDS hash table,
    //      the K negatives are streamed past it, every hit bumps the count of its slot
    if (p.cnt) {
        for (int s = tid; s < kTgtSlots; s += kPrepThreads) {
            hkey[s] = -1;
            hcnt[s] = 0;
        }
        __syncthreads();
        int my_slot = -1;
        if (valid) {
            uint32_t h = hash_id(ti, kTgtSlots);
            for (int probe = 0; probe < kTgtSlots; ++probe) {
                const int32_t prev = atomicCAS(&hkey[h], -1, ti);
                if (prev == -1 || prev == ti) {
                    my_slot = (int)h;
                    break;
                }
                h = (h + 1) & (kTgtSlots - 1);
            }
        }
        __syncthreads();
        for (int64_t k = tid; k < p.K; k += kPrepThreads) {
            const int32_t id = p.neg[k];
            if (id < 0) continue;  // flagged by the range check below; never equal to a valid target
            uint32_t h = hash_id(id, kTgtSlots);
            for (int probe = 0; probe < kTgtSlots; ++probe) {
                const int32_t key = hkey[h];
                if (key == id) {
                    atomicAdd(&hcnt[h], 1);
                    break;
                }
                if (key == -1) break;
                h = (h + 1) & (kTgtSlots - 1);
            }
        }
        __syncthreads();
        if (valid) p.cnt[i] = hcnt[my_slot];
    }

    // ---- range check of the shared negatives (once, by block 0)
    if (p.validate && p.neg && blockIdx.x == 0) {
        bool bad = false;
        for (int64_t k = tid; k < p.K; k += kPrepThreads) {
            const int32_t id = p.neg[k];
            bad |= (id < 0 || (int64_t)id >= p.V);
        }
        if (bad) atomicOr(p.header + kHdrStatus, 1);
    }
}

// ---------------------------------------------------------------------------------------------------------------------
// Merges of split runs (few positions, many candidates: the candidate range is split over blocks).
template <int D>
__global__ __launch_bounds__(256) void fwd_merge_kernel(TileArgs a)
{
    // 8 lanes per position: each takes the chunks c, c+8, ... of the row for the correct-item score
    const int64_t n_pos = a.n_valid_ptr ? (int64_t)*a.n_valid_ptr : a.N;
    const int64_t x = ((int64_t)blockIdx.x * 256 + threadIdx.x) / 8;
    const int c = threadIdx.x & 7;
    const bool ok = x < n_pos;
    const int64_t row = ok ? pos_row(a, x) : 0;
    float op = 0.f;
    if (ok) {
        const uint16_t *hp = a.H + row * D, *ep = a.E + (int64_t)a.tgt[row] * D;
        for (int ch = c; ch < D / 8; ch += 8) {
            float h[8], e[8];
            load8(hp + ch * 8, h);
            load8(ep + ch * 8, e);
#pragma unroll
            for (int t = 0; t < 8; ++t) op = fmaf(h[t], e[t], op);
        }
    }
    op += __shfl_xor(op, 1, 64);
    op += __shfl_xor(op, 2, 64);
    op += __shfl_xor(op, 4, 64);
    if (ok && c == 0) {
        float m = -INFINITY, s = 0.f;
        for (int sp = 0; sp < a.splits; ++sp) {
            const float m2 = a.part_m[(int64_t)sp * a.N + x], s2 = a.part_s[(int64_t)sp * a.N + x];
            const float M = fmaxf(m, m2);
            if (M > -INFINITY) {
                s = s * __builtin_amdgcn_exp2f(m - M) + s2 * __builtin_amdgcn_exp2f(m2 - M);
                m = M;
            }
        }
        const float w = a.pos_weight_mode == 2 ? 0.f : (a.cnt ? 1.f - (float)a.cnt[row] : 1.f);
        const float o2 = op * kLog2e;
        const float M = (w != 0.f) ? fmaxf(m, o2) : m;
        const float tot = s * __builtin_amdgcn_exp2f(m - M) + w * __builtin_amdgcn_exp2f(o2 - M);
        const float l = (M + __builtin_amdgcn_logf(tot)) * kLn2;
        a.lse[row] = l;
        a.loss[row] = l - op;
    }
}

template <int D>
__global__ __launch_bounds__(256) void dh_merge_kernel(TileArgs a)
{
    constexpr int LPR = D / 8;  // lanes per position, 8 columns each
    static_assert(64 % LPR == 0 || LPR % 64 == 0, "row must tile the wavefront");
    constexpr int PPB = 256 / LPR;
    const int64_t n_pos = a.n_valid_ptr ? (int64_t)*a.n_valid_ptr : a.N;
    const int64_t x = (int64_t)blockIdx.x * PPB + threadIdx.x / LPR;
    const int c = threadIdx.x % LPR;
    const bool ok = x < n_pos;
    const int64_t row = ok ? pos_row(a, x) : 0;
    float h[8], e[8], sum[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) h[t] = e[t] = sum[t] = 0.f;
    float op = 0.f;
    if (ok) {
        load8(a.H + row * D + c * 8, h);
        load8(a.E + (int64_t)a.tgt[row] * D + c * 8, e);
#pragma unroll
        for (int t = 0; t < 8; ++t) op = fmaf(h[t], e[t], op);
        for (int sp = 0; sp < a.splits; ++sp) {
            float v[8];
            load8(a.part_dH + ((int64_t)sp * a.N + x) * D + c * 8, v);
#pragma unroll
            for (int t = 0; t < 8; ++t) sum[t] += v[t];
        }
    }
    // rows never straddle a wavefront when LPR <= 64; for D = 512 this kernel is not instantiated
#pragma unroll
    for (int off = 1; off < LPR && off < 64; off <<= 1) op += __shfl_xor(op, off, 64);
    if (ok) {
        const float w = a.pos_weight_mode == 2 ? 0.f : (a.cnt ? 1.f - (float)a.cnt[row] : 1.f);
        const float pp = __builtin_amdgcn_exp2f((op - a.lse_in[row]) * kLog2e);
        const float cpos = w * pp - 1.f;
        const float g = a.g ? a.g[row] : 1.f;
        if (c == 0) a.coef[row] = g * cpos;
        float v[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] = g * fmaf(cpos, e[t], sum[t]);
        if (a.dH_bf16) {
            *reinterpret_cast<uint4 *>(static_cast<uint16_t *>(a.dH) + row * D + c * 8) =
                make_uint4(pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7]));
        } else {
            float4 *out = reinterpret_cast<float4 *>(static_cast<float *>(a.dH) + row * D + c * 8);
            out[0] = make_float4(v[0], v[1], v[2], v[3]);
            out[1] = make_float4(v[4], v[5], v[6], v[7]);
        }
    }
}

// ---------------------------------------------------------------------------------------------------------------------
// dE of the correct items: dE[tgt_i] += coef_i * H_i.  Targets follow a power law, so plain atomics would serialise
// on a few hot rows.  Each block counts its 256 targets in an LDS hash table; a target met once is added straight
// away (one wavefront per row, consecutive addresses), a target met several times has its positions gathered into a
// segment that one wavefront sums in registers before a single atomic row add.
constexpr int kPosChunk = 256;
constexpr int kPosSlots = 512;

template <int D>
__global__ __launch_bounds__(256) void pos_scatter_kernel(TileArgs a)
{
    constexpr int CPL = D / 64;  // columns per lane: lane owns columns lane*CPL .. +CPL of a row
    __shared__ int32_t hkey[kPosSlots];
    __shared__ int32_t hcnt[kPosSlots];
    __shared__ int32_t hoff[kPosSlots];
    __shared__ int32_t hcur[kPosSlots];
    __shared__ int32_t grouped[kPosChunk];   // position rows of the repeated targets, segment after segment
    __shared__ int32_t seg_key[kPosChunk / 2], seg_off[kPosChunk / 2], seg_len[kPosChunk / 2];
    __shared__ int32_t n_grouped, n_segs;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t n_pos = a.n_valid_ptr ? (int64_t)*a.n_valid_ptr : a.N;
    const int64_t e = (int64_t)blockIdx.x * kPosChunk + tid;
    if ((int64_t)blockIdx.x * kPosChunk >= n_pos) return;
    const bool have = e < n_pos;
    const int32_t row = have ? (int32_t)pos_row(a, e) : -1;
    const int32_t key = have ? a.tgt[row] : -1;

    for (int s = tid; s < kPosSlots; s += 256) {
        hkey[s] = -1;
        hcnt[s] = 0;
        hcur[s] = 0;
    }
    if (tid == 0) {
        n_grouped = 0;
        n_segs = 0;
    }
    __syncthreads();
    int slot = -1;
    bool leader = false;
    if (have) {
        uint32_t h = hash_id(key, kPosSlots);
        for (int probe = 0; probe < kPosSlots; ++probe) {
            const int32_t prev = atomicCAS(&hkey[h], -1, key);
            if (prev == -1 || prev == key) {
                slot = (int)h;
                leader = (prev == -1);
                atomicAdd(&hcnt[h], 1);
                break;
            }
            h = (h + 1) & (kPosSlots - 1);
        }
    }
    __syncthreads();
    const int n_same = have ? hcnt[slot] : 0;
    if (leader && n_same > 1) {
        const int off = atomicAdd(&n_grouped, n_same);
        const int sg = atomicAdd(&n_segs, 1);
        hoff[slot] = off;
        seg_key[sg] = key;
        seg_off[sg] = off;
        seg_len[sg] = n_same;
    }
    __syncthreads();
    if (n_same > 1) grouped[hoff[slot] + atomicAdd(&hcur[slot], 1)] = row;
    __syncthreads();

    // ---- targets met once: the wavefront walks over its lanes' entries, four rows in flight
    {
        uint64_t todo = __ballot(n_same == 1);
        while (todo) {
            int32_t r4[4], k4[4];
            float c4[4];
            float h4[4][CPL];
            int n = 0;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                r4[u] = -1;
                if (todo) {
                    const int src = __ffsll((unsigned long long)todo) - 1;
                    todo &= todo - 1;
                    r4[u] = __shfl(row, src, 64);
                    k4[u] = __shfl(key, src, 64);
                    n = u + 1;
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (u < n) {
                    c4[u] = a.coef[r4[u]];
#pragma unroll
                    for (int t = 0; t < CPL; ++t) h4[u][t] = load1(a.H + (int64_t)r4[u] * D + lane * CPL + t);
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (u < n) {
#pragma unroll
                    for (int t = 0; t < CPL; ++t)
                        unsafeAtomicAdd(a.dE + (int64_t)k4[u] * D + lane * CPL + t, c4[u] * h4[u][t]);
                }
            }
        }
    }
    // ---- repeated targets: one wavefront per segment
    const int segs = n_segs;
    for (int sg = wave; sg < segs; sg += 4) {
        const int off = seg_off[sg], len = seg_len[sg];
        float accv[CPL];
#pragma unroll
        for (int t = 0; t < CPL; ++t) accv[t] = 0.f;
        for (int j0 = 0; j0 < len; j0 += 4) {
            float c4[4];
            float h4[4][CPL];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                c4[u] = 0.f;
#pragma unroll
                for (int t = 0; t < CPL; ++t) h4[u][t] = 0.f;
                if (j0 + u < len) {
                    const int32_t r = grouped[off + j0 + u];
                    c4[u] = a.coef[r];
#pragma unroll
                    for (int t = 0; t < CPL; ++t) h4[u][t] = load1(a.H + (int64_t)r * D + lane * CPL + t);
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int t = 0; t < CPL; ++t) accv[t] = fmaf(c4[u], h4[u][t], accv[t]);
        }
        const int64_t k = seg_key[sg];
#pragma unroll
        for (int t = 0; t < CPL; ++t) unsafeAtomicAdd(a.dE + k * D + lane * CPL + t, accv[t]);
    }
}

// ---------------------------------------------------------------------------------------------------------------------
template <int D>
hipError_t launch_for_d(int pass, const TileArgs &a, hipStream_t stream)
{
    constexpr int BY = (D <= 128) ? 64 : 32;
    const int64_t n_x = (pass == TILE_PASS_DE) ? a.n_cols : a.N;
    const int64_t xblocks = (n_x + kXPerBlock - 1) / kXPerBlock;
    if (xblocks == 0) return hipSuccess;
    const dim3 grid((unsigned)(xblocks * a.splits)), block(kThreads);
    switch (pass) {
    case TILE_PASS_FWD:
        hipLaunchKernelGGL((tile_kernel<D, MODE_FWD, BY>), grid, block, 0, stream, a);
        if (a.splits > 1)
            hipLaunchKernelGGL((fwd_merge_kernel<D>), dim3((unsigned)((a.N * 8 + 255) / 256)), dim3(256), 0, stream, a);
        break;
    case TILE_PASS_DH:
        hipLaunchKernelGGL((tile_kernel<D, MODE_DH, BY>), grid, block, 0, stream, a);
        if (a.splits > 1) {
            constexpr int PPB = 256 / (D / 8);
            hipLaunchKernelGGL((dh_merge_kernel<D>), dim3((unsigned)((a.N + PPB - 1) / PPB)), dim3(256), 0, stream, a);
        }
        break;
    case TILE_PASS_DE:
        hipLaunchKernelGGL((tile_kernel<D, MODE_DE, BY>), grid, block, 0, stream, a);
        break;
    case TILE_PASS_POS:
        hipLaunchKernelGGL((pos_scatter_kernel<D>), dim3((unsigned)((a.N + kPosChunk - 1) / kPosChunk)), dim3(256), 0,
                           stream, a);
        break;
    default:
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

bool tile_supports_d(int d) { return d == 64 || d == 128 || d == 256; }

hipError_t launch_prep(const PrepArgs &p, hipStream_t stream)
{
    if (p.N == 0) return hipSuccess;
    hipLaunchKernelGGL(prep_kernel, dim3((unsigned)((p.N + kPrepThreads - 1) / kPrepThreads)), dim3(kPrepThreads), 0,
                       stream, p);
    return hipGetLastError();
}

hipError_t launch_tile(int pass, const TileArgs &a, hipStream_t stream)
{
    if (a.N == 0) return hipSuccess;
    switch (a.d) {
    case 64: return launch_for_d<64>(pass, a, stream);
    case 128: return launch_for_d<128>(pass, a, stream);
    case 256: return launch_for_d<256>(pass, a, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace cce
