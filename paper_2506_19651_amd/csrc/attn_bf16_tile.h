// Tile-level building blocks of the bf16 MFMA attention kernels (gfx950): staging layout of a key
// tile in LDS, S^T = K Q^T and O^T += V^T P^T on v_mfma_f32_32x32x16_bf16, masks, the weights of the
// online softmax.  Shared by the one-item-per-workgroup kernel and the streaming kernel.
#pragma once
#include "bf16_device.h"

namespace pevlm {

template <int D>
struct TileCfg {
    static constexpr int KT = kKeyTile;        // keys per staged tile
    static constexpr int ROWB = D * 2;         // bytes per K/V row
    static constexpr int CH = D / 8;           // 16-byte chunks per row
    static constexpr int NLD = KT * CH / 256;  // 16-byte loads each wavefront issues per tensor per tile
    static constexpr int KSTEPS = D / 16;      // MFMA k-steps of Q K^T
    static constexpr int DBLK = D / 32;        // 32-wide blocks of head_dim in O^T
    static constexpr int VSW = CH / 4 - 1;     // V swizzle mask (64-byte granules per row - 1)
    static constexpr int TILEB = KT * ROWB;    // bytes of one staged K (or V) tile
    static constexpr int RPI = 1024 / ROWB;    // rows one wavefront-wide 16-byte-per-lane load covers
};

// per-lane LDS offsets (the XOR swizzles depend on the lane only)
struct LaneOff {
    int32_t k_row_off, k_swz, v_row_off, v_ch_lo, v_swz, g32;
};

// Global->LDS loads a wavefront slips between the MFMAs of a tile (its share of the next K tile
// during the score MFMAs, of the current V tile during the value MFMAs): a wavefront-uniform base
// address, per-lane byte offsets and the LDS address of the wave's first 1 KB piece.
template <int NLD>
struct TileLoads {
    const void *base;
    uint32_t off[NLD > 0 ? NLD : 1];
    uint32_t lds;
};
// The wave's j-th 1 KB piece of a tile lies PSTEP bytes after its (j-1)-th: 4 wavefronts share a tile
// in the one-item kernel (4 KB), 8 in the streaming kernel (8 KB).

constexpr float kRescaleStep = 8.f;  // log2 units the row maximum may outgrow the reference maximum

// S^T = K Q^T for the 64 keys of a staged tile: two independent accumulation chains (one per
// 32-key chunk) issued alternately; A fragments (16 bytes per lane) are fetched half a tile ahead.
template <int D, bool LOADS, int NL = D / 32, int PSTEP = 4096>
__device__ __forceinline__ void qk_tile(const uint8_t *tk, const LaneOff &L, const bf16x8 (&qf)[D / 16], f32x16 (&s)[2],
                                        const TileLoads<NL> &ld)
{
    using C = TileCfg<D>;
    constexpr int HK = C::KSTEPS / 2;
    const f32x16 init = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    bf16x8 a0[C::KSTEPS], a1[C::KSTEPS];
#define PEVLM_KFRAG(kc, kk) \
    (*reinterpret_cast<const bf16x8 *>(tk + (kc) * 32 * C::ROWB + L.k_row_off + ((((kk) * 2 + L.g32) ^ L.k_swz) << 4)))
#pragma unroll
    for (int kk = 0; kk < HK; ++kk) {
        a0[kk] = PEVLM_KFRAG(0, kk);
        a1[kk] = PEVLM_KFRAG(1, kk);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < HK; ++kk) {
        s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[kk], qf[kk], kk == 0 ? init : s[0], 0, 0, 0);
        a0[kk + HK] = PEVLM_KFRAG(0, kk + HK);
        s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[kk], qf[kk], kk == 0 ? init : s[1], 0, 0, 0);
        a1[kk + HK] = PEVLM_KFRAG(1, kk + HK);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = HK; kk < C::KSTEPS; ++kk) {
        s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[kk], qf[kk], s[0], 0, 0, 0);
        s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[kk], qf[kk], s[1], 0, 0, 0);
        if (LOADS && kk - HK < NL) {  // one 1 KB piece of a later K tile per pair of MFMAs
            load_lds_16_base(ld.base, ld.off[kk - HK < NL ? kk - HK : 0], ld.lds + (kk - HK) * PSTEP);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#undef PEVLM_KFRAG
}

// Same scores with the A fragments fetched only PF k-steps ahead of their MFMAs (a ring of PF
// fragments per 32-key chunk instead of half a tile): fewer live registers, for the kernel that has
// none to spare.  `ld.issue(j)` requests the wavefront's j-th piece (of NL) of a later K tile.
template <int D, bool LOADS, int NL, class LD, int PF = 2>
__device__ __forceinline__ void qk_tile_ring(const uint8_t *tk, const LaneOff &L, const bf16x8 (&qf)[D / 16], f32x16 (&s)[2],
                                             const LD &ld)
{
    using C = TileCfg<D>;
    constexpr int KS = C::KSTEPS, HK = KS / 2;
    const f32x16 init = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    bf16x8 a0[KS], a1[KS];
#define PEVLM_KFRAG(kc, kk) \
    (*reinterpret_cast<const bf16x8 *>(tk + (kc) * 32 * C::ROWB + L.k_row_off + ((((kk) * 2 + L.g32) ^ L.k_swz) << 4)))
#pragma unroll
    for (int kk = 0; kk < PF; ++kk) {
        a0[kk] = PEVLM_KFRAG(0, kk);
        a1[kk] = PEVLM_KFRAG(1, kk);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
        s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[kk], qf[kk], kk == 0 ? init : s[0], 0, 0, 0);
        if (kk + PF < KS) a0[kk + PF] = PEVLM_KFRAG(0, kk + PF);
        s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[kk], qf[kk], kk == 0 ? init : s[1], 0, 0, 0);
        if (kk + PF < KS) a1[kk + PF] = PEVLM_KFRAG(1, kk + PF);
        if (LOADS && kk >= HK && kk - HK < NL) ld.issue(kk - HK);  // one 1 KB piece of a later K tile per pair of MFMAs
        __builtin_amdgcn_sched_barrier(0);
    }
#undef PEVLM_KFRAG
}

// V^T fragments of 16 keys (k-step ks of the staged tile) for every 32-wide block of head_dim
template <int D>
__device__ __forceinline__ void read_v(const uint8_t *tv, const LaneOff &L, int ks, bf16x8 (&dst)[D / 32])
{
    using C = TileCfg<D>;
#pragma unroll
    for (int b = 0; b < C::DBLK; ++b)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            const uint8_t *ptr = tv + (ks * 16 + tt * 8) * C::ROWB + L.v_row_off + (((b ^ L.v_swz) * 4 + L.v_ch_lo) << 4);
            const s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, ptr));
            const bf16x4 rb = __builtin_bit_cast(bf16x4, r);
            dst[b][tt * 4 + 0] = rb[0]; dst[b][tt * 4 + 1] = rb[1];
            dst[b][tt * 4 + 2] = rb[2]; dst[b][tt * 4 + 3] = rb[3];
        }
}

// entries a row must not see: beyond the key range, or (causal range) keys after the row.  Key
// k0 + c is visible iff c <= min(kend - 1, causal ? my_row : inf) - k0; c = const + 4*g32 per entry,
// so each entry costs one compare against a per-lane limit and one select.
__device__ __forceinline__ void mask_tile(f32x16 (&s)[2], int32_t k0, int32_t kend, bool causal, int32_t my_row, int32_t g32)
{
    int32_t last = kend - 1;
    if (causal) last = my_row < last ? my_row : last;
    const int32_t lim = last - k0 - g32 * 4;
#pragma unroll
    for (int kc = 0; kc < 2; ++kc)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int32_t c = kc * 32 + (i >> 2) * 8 + (i & 3);
            s[kc][i] = c <= lim ? s[kc][i] : -INFINITY;
        }
}

// maximum over the 64 keys of the tile for this lane's row (both lanes of a row end up with it)
__device__ __forceinline__ float row_max(const f32x16 (&s)[2])
{
    float mx = max3f(s[0][0], s[0][1], s[0][2]);
#pragma unroll
    for (int i = 3; i < 31; i += 2) mx = max3f(mx, s[i >> 4][i & 15], s[(i + 1) >> 4][(i + 1) & 15]);
    mx = fmaxf(mx, s[1][15]);
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
    return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}

// weights p = exp2(c s - m) of the tile (c = scale*log2(e), m = the row's reference maximum in
// base-2 units): bf16 pairs (B fragments of the value MFMAs) and their sum over this lane's 32 keys
// (dot product of each pair with (1, 1)).  Weights are non-negative, so a sum below 2^kRescaleStep
// bounds every one of them; an overflowed or invalid weight makes the sum inf or nan.
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__device__ __forceinline__ uint32_t weight_pair(float s0, float s1, float c_log2, float mref, float &psum)
{
    bf16x2 pr;
    pr[0] = (__bf16)__builtin_amdgcn_exp2f(s0 * c_log2 - mref);
    pr[1] = (__bf16)__builtin_amdgcn_exp2f(s1 * c_log2 - mref);
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    psum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, psum, false);
    return __builtin_bit_cast(uint32_t, pr);
}

__device__ __forceinline__ void weights(const f32x16 (&s)[2], float c_log2, float mref, float &psum, u32x4 (&pf)[4])
{
#pragma unroll
    for (int kc = 0; kc < 2; ++kc)
#pragma unroll
        for (int i = 0; i < 16; i += 2) pf[kc * 2 + (i >> 3)][(i & 7) >> 1] = weight_pair(s[kc][i], s[kc][i + 1], c_log2, mref, psum);
}

// true unless this lane's sum of weights proves that all of them stayed below 2^kRescaleStep
__device__ __forceinline__ bool sum_reached_step(float psum) { return !(psum < 256.f); }
static_assert(kRescaleStep == 8.f, "sum_reached_step compares with 2^kRescaleStep");

// O^T += V^T P^T for a staged V tile (16 MFMAs per 32 values of head_dim ... 4 k-steps x DBLK blocks)
template <int D>
__device__ __forceinline__ void pv_tile(const uint8_t *tv, const LaneOff &L, const u32x4 (&pf)[4], f32x16 (&o)[D / 32])
{
    using C = TileCfg<D>;
    bf16x8 va[C::DBLK], vb[C::DBLK];
    read_v<D>(tv, L, 0, va);
#pragma unroll
    for (int ks = 0; ks < 4; ks += 2) {
        read_v<D>(tv, L, ks + 1, vb);
#pragma unroll
        for (int b = 0; b < C::DBLK; ++b) o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[b], __builtin_bit_cast(bf16x8, pf[ks]), o[b], 0, 0, 0);
        if (ks + 2 < 4) read_v<D>(tv, L, ks + 2, va);
#pragma unroll
        for (int b = 0; b < C::DBLK; ++b) o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vb[b], __builtin_bit_cast(bf16x8, pf[ks + 1]), o[b], 0, 0, 0);
    }
}

// One V^T fragment: 16 keys (k-step ks) x the b-th 32-wide block of head_dim
template <int D>
__device__ __forceinline__ bf16x8 read_v_one(const uint8_t *tv, const LaneOff &L, int ks, int b)
{
    using C = TileCfg<D>;
    bf16x8 dst;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
        const uint8_t *ptr = tv + (ks * 16 + tt * 8) * C::ROWB + L.v_row_off + (((b ^ L.v_swz) * 4 + L.v_ch_lo) << 4);
        const s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, ptr));
        const bf16x4 rb = __builtin_bit_cast(bf16x4, r);
        dst[tt * 4 + 0] = rb[0]; dst[tt * 4 + 1] = rb[1];
        dst[tt * 4 + 2] = rb[2]; dst[tt * 4 + 3] = rb[3];
    }
    return dst;
}

// The pipelined step: O^T += V^T P^T of the previous tile (matrix cores) issued one MFMA at a time,
// each followed by the vector-ALU work for a pair (or two) of weights of the current tile, so that
// both pipes of the SIMD run from one instruction stream.  V^T fragments are read one k-step ahead.
template <int D, int NL = D / 32, int PSTEP = 4096>
__device__ __forceinline__ void pv_prev_weights_cur(const uint8_t *tv_prev, const LaneOff &L, const u32x4 (&pf_prev)[4],
                                                    f32x16 (&o)[D / 32], const f32x16 (&s)[2], float c_log2,
                                                    float mref, float &psum, u32x4 (&pf_new)[4], const TileLoads<NL> &ld)
{
    using C = TileCfg<D>;
    constexpr int NM = 4 * C::DBLK;  // MFMAs of the tile
    constexpr int PPM = 16 / NM;     // weight pairs formed per MFMA
    bf16x8 vf[2][C::DBLK];
#pragma unroll
    for (int b = 0; b < C::DBLK; ++b) vf[0][b] = read_v_one<D>(tv_prev, L, 0, b);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int n = 0; n < NM; ++n) {
        const int ks = n / C::DBLK, b = n % C::DBLK;
        if (ks + 1 < 4) vf[(ks + 1) & 1][b] = read_v_one<D>(tv_prev, L, ks + 1, b);
        o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[ks & 1][b], __builtin_bit_cast(bf16x8, pf_prev[ks]), o[b], 0, 0, 0);
        if (n % 4 == 0 && n / 4 < NL) load_lds_16_base(ld.base, ld.off[n / 4 < NL ? n / 4 : 0], ld.lds + (n / 4) * PSTEP);  // a piece of a V tile
#pragma unroll
        for (int e = 0; e < PPM; ++e) {
            const int pi = n * PPM + e, kc = pi >> 3, i = (pi & 7) * 2;
            pf_new[kc * 2 + (i >> 3)][(i & 7) >> 1] = weight_pair(s[kc][i], s[kc][i + 1], c_log2, mref, psum);
        }
        // keep the running values here (plain arithmetic would otherwise be emitted after the last MFMA)
        asm volatile("" : "+v"(psum));
        if (((n + 1) * PPM) % 4 == 0) asm volatile("" : "+v"(pf_new[((n + 1) * PPM) / 4 - 1]));
        __builtin_amdgcn_sched_barrier(0);
    }
}

// The same pipelined step with the V^T fragments fetched only PF MFMAs ahead (a ring of PF fragments
// instead of two k-steps of them): fewer live registers.  `ld.issue(j)` requests the wavefront's j-th
// piece (of NL) of a later V tile.
template <int D, int NL, class LD, int PF = 3>
__device__ __forceinline__ void pv_prev_weights_cur_ring(const uint8_t *tv_prev, const LaneOff &L, const u32x4 (&pf_prev)[4],
                                                         f32x16 (&o)[D / 32], const f32x16 (&s)[2], float c_log2,
                                                         float mref, float &psum, u32x4 (&pf_new)[4], const LD &ld)
{
    using C = TileCfg<D>;
    constexpr int NM = 4 * C::DBLK;  // MFMAs of the tile
    constexpr int PPM = 16 / NM;     // weight pairs formed per MFMA
    bf16x8 vf[NM];
#pragma unroll
    for (int n = 0; n < PF; ++n) vf[n] = read_v_one<D>(tv_prev, L, n / C::DBLK, n % C::DBLK);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int n = 0; n < NM; ++n) {
        const int ks = n / C::DBLK, b = n % C::DBLK;
        if (n + PF < NM) vf[n + PF] = read_v_one<D>(tv_prev, L, (n + PF) / C::DBLK, (n + PF) % C::DBLK);
        o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[n], __builtin_bit_cast(bf16x8, pf_prev[ks]), o[b], 0, 0, 0);
        if (n % 4 == 0 && n / 4 < NL) ld.issue(n / 4);
#pragma unroll
        for (int e = 0; e < PPM; ++e) {
            const int pi = n * PPM + e, kc = pi >> 3, i = (pi & 7) * 2;
            pf_new[kc * 2 + (i >> 3)][(i & 7) >> 1] = weight_pair(s[kc][i], s[kc][i + 1], c_log2, mref, psum);
        }
        asm volatile("" : "+v"(psum));
        if (((n + 1) * PPM) % 4 == 0) asm volatile("" : "+v"(pf_new[((n + 1) * PPM) / 4 - 1]));
        __builtin_amdgcn_sched_barrier(0);
    }
}

}  // namespace pevlm
