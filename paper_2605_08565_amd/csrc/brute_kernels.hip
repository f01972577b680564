// Brute-force scale search (last paragraph of Section 2): for every block, every finite,
// strictly positive scale code is tried; the code of minimal block SSE wins, the lowest code
// on a tie.  Same lane mapping as the streaming kernels (8 elements per lane).  The tensor is
// read once and every candidate costs only ALU work, so this kernel is bound by the fp32
// vector units, not by HBM.
//
// A scale is S = m * 2^e with m in {1, 1.125, .., 1.875}.  Dividing by 2^e commutes with
// rounding, so the quotient v / S is formed once per mantissa (w_m = v / m, 7 divisions per
// element instead of one per candidate) and the E2M1 conversion instruction applies 2^e.
// The inverse conversion returns q * 2^e, and the residual v - (q * 2^e) * m needs a single
// FMA because the product is exact.  Candidates are visited in ascending code order, one
// binade (8 codes) at a time, so a strict "less than" between binades and the first position
// inside one keep the lowest code on ties.
//
// Power-of-two scales (E8M0, every byte 0x00 .. 0xFE is a finite positive value, 255 candidates)
// need no quotient at all: the conversion instruction divides by 2^k itself.
#include "mxq_device.hpp"
#include "mxq_launch.hpp"

namespace mxq {

// hi/lo split of 1/m for m = 1 + i/8 (see "Quotients whose rounding decisions are exact").
__device__ constexpr float mant_value(int i) { return 1.0f + (float)i * 0.125f; }
__device__ constexpr float mant_rhi(int i)                          // 1/m rounded toward zero
{
    const double d = 1.0 / (1.0 + i * 0.125);
    const float r = (float)d;
    return ((double)r > d) ? __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, r) - 1u) : r;
}
__device__ constexpr float mant_rlo(int i) { return (float)(1.0 / (1.0 + i * 0.125) - (double)mant_rhi(i)); }

template <int B>
struct BruteState {
    static constexpr int NBLK = (B < 8) ? 8 / B : 1;
    float best_sse[NBLK];
    uint32_t best_code[NBLK];
};

// Arg-min over a group of up to 8 consecutive codes (one binade): begin(), put<POS>(k, sse) per
// candidate and block slot, end(st, code0) -- the code of position p is code0 + p.  The
// candidates only deposit their block SSEs; the group's minimum (three-input minimum
// instructions) is compared with the running best once per group, and only when some lane of
// the wavefront improved is the position of the minimum looked up (the first position that
// equals it: the lowest code on a tie inside the group; between groups "strictly less" keeps
// the earlier, lower code).  A candidate costs half an instruction here; measured against a
// compare and two selects per candidate it is faster also when most groups improve (the
// pruned search).
template <int B>
struct GroupArgMin {
    static constexpr int NBLK = BruteState<B>::NBLK;
    float s[NBLK][8];

    // Position 7 is the only one that can be without a candidate (the 7 sub-normal codes; the
    // NaN code at the top of the last binade): +inf never wins.
    __device__ __forceinline__ void begin()
    {
#pragma unroll
        for (int k = 0; k < NBLK; ++k) s[k][7] = __builtin_inff();
    }
    template <int POS>
    __device__ __forceinline__ void put(int k, float sse) { s[k][POS] = sse; }
    // Take position 7 of block slot k out of this group (the code there is not a number).
    __device__ __forceinline__ void drop_last(int k, bool drop) { s[k][7] = drop ? __builtin_inff() : s[k][7]; }

    __device__ __forceinline__ void end(BruteState<B>& st, uint32_t code0) const
    {
        uint32_t c0[NBLK];
        bool ok[NBLK];
#pragma unroll
        for (int k = 0; k < NBLK; ++k) { c0[k] = code0; ok[k] = true; }
        end(st, c0, ok);
    }
    // code0 per block slot; a slot with ok == false takes no part in this group
    __device__ __forceinline__ void end(BruteState<B>& st, const uint32_t (&code0)[NBLK], const bool (&ok)[NBLK]) const
    {
        float gmin[NBLK];
        bool any = false;
#pragma unroll
        for (int k = 0; k < NBLK; ++k) {
            const float a = fminf(fminf(s[k][0], s[k][1]), s[k][2]);
            const float b = fminf(fminf(s[k][3], s[k][4]), s[k][5]);
            gmin[k] = fminf(fminf(a, b), fminf(s[k][6], s[k][7]));
            any |= ok[k] && gmin[k] < st.best_sse[k];
        }
        if (__builtin_amdgcn_ballot_w64(any) == 0ull) return;           // wave-uniform
#pragma unroll
        for (int k = 0; k < NBLK; ++k) {
            uint32_t pos = 7u;
#pragma unroll
            for (int i = 6; i >= 0; --i) pos = (s[k][i] == gmin[k]) ? (uint32_t)i : pos;
            const bool better = ok[k] && gmin[k] < st.best_sse[k];
            st.best_code[k] = better ? code0[k] + pos : st.best_code[k];
            st.best_sse[k] = better ? gmin[k] : st.best_sse[k];
        }
    }
};

// SSE of the lane's blocks under S = mant_value(MI) * scale2 (scale2 a power of two), entered
// into the group at position POS.  w holds the lane's quotients v / mant_value(MI).
template <int B, int MI, int POS, class G>
__device__ __forceinline__ void try_candidate(const float (&v)[8], const float (&w)[8], float scale2, G& g)
{
    const uint32_t packed = e2m1_pack8(w, scale2);
    float q2[8], sq[8];
    e2m1_unpack8(packed, scale2, q2);                                  // q * 2^e
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        float e;
        if constexpr (MI == 0) e = v[j] - q2[j];
        else e = __builtin_fmaf(-q2[j], mant_value(MI), v[j]);
        sq[j] = e * e;
    }
    const float p0 = sq[0] + sq[1], p1 = sq[2] + sq[3], p2 = sq[4] + sq[5], p3 = sq[6] + sq[7];
    if constexpr (B == 2) {
        g.template put<POS>(0, p0); g.template put<POS>(1, p1);
        g.template put<POS>(2, p2); g.template put<POS>(3, p3);
    } else if constexpr (B == 4) {
        g.template put<POS>(0, p0 + p1); g.template put<POS>(1, p2 + p3);
    } else {
        g.template put<POS>(0, group_sum<B / 8>((p0 + p1) + (p2 + p3)));
    }
    // One candidate at a time: left alone, the instruction scheduler interleaves several
    // candidates, which costs registers and 10 % of the kernel's speed (measured).
    __builtin_amdgcn_sched_barrier(0);
}

template <int B, int FMT, int MI, class G>
__device__ __forceinline__ void try_binade_from(const float (&v)[8], const float (&w)[8][8], float scale2,
                                                uint32_t code0, G& g)
{
    if constexpr (MI < 7) {
        try_candidate<B, MI, MI>(v, w[MI], scale2, g);
        try_binade_from<B, FMT, MI + 1>(v, w, scale2, code0, g);
    } else {
        if (code0 + 7u <= (uint32_t)ScaleFmt<FMT>::kMaxCode)            // skips the NaN code only
            try_candidate<B, 7, 7>(v, w[7], scale2, g);
    }
}

// The 8 codes code0 .. code0 + 7 of one binade: (1 + mi/8) * scale2.
template <int B, int FMT>
__device__ __forceinline__ void try_binade(const float (&v)[8], const float (&w)[8][8], float scale2,
                                           uint32_t code0, BruteState<B>& st)
{
    GroupArgMin<B> g;
    g.begin();
    try_binade_from<B, FMT, 0>(v, w, scale2, code0, g);
    g.end(st, code0);
}

// ---------------------------------------------------------------------------------------
// Pruned search (recipe BRUTE_PRUNED): same result as the full enumeration, bit for bit,
// fewer candidates.  Three facts bound the useful codes of a block with abs-max `amax`:
//   (hi) S >= 4*amax quantises every element to zero, so all such candidates share one SSE
//        (sum of squares); the first of them has the lowest code, the others can only tie.
//   (hi2) under any scale S >= S0 an element with |v| < S0/2 quantises to 0 or to S/2, with a
//        residual of |v| or of S/2 - |v| >= S0/2 - |v| > 0, so its square in the SSE is at least
//        min(fl(v^2), fl(fl(S0/2 - |v|)^2)) (for |v| < S0/4, where it is certain to vanish, that is
//        fl(v^2) itself); the other elements contribute >= +0, and an fp32 sum of non-negative
//        terms does not fall when a term grows.  The tree sum of these terms is therefore a lower
//        bound of the SSE of every scale >= S0; it grows with S0, and once it exceeds U (below)
//        every higher code loses.  On weights this ends the window two binades above the abs-max
//        scale, where (hi) alone lets it run to five or six.
//   (lo) while 6*S < amax the abs-max element saturates and alone contributes
//        fl(fl(amax - 6S)^2); fp32 sums of non-negative terms never fall below a term, so that
//        is a lower bound of the candidate's SSE.  Once it exceeds U, the SSE of a reference
//        candidate (the abs-max scale), the candidate cannot win; the bound falls with S, so
//        the losers form a prefix of the code range (tested per binade, bisection as fall-back).
// Windows of different blocks sit at different places of the code range (wherever the block's
// abs-max puts them) but have nearly the same width, about one binade below the abs-max scale to
// two or three above ((hi) alone: five to six).  So the scan is wave-uniform in RELATIVE terms:
// in step t every block tries the t-th binade of its OWN window (the power of two handed to the
// conversion instruction is a per-lane register, the mantissa stays uniform), t running up to
// the widest window of the wavefront.  A wavefront with 128 small blocks then visits hardly more
// candidates than its widest block alone would, where a scan of the union of the absolute
// windows degrades with the number of blocks per wavefront and with the spread of their
// magnitudes.  Lanes whose window has ended are masked out; the sub-normal codes are one uniform
// group in front.  Every block visits its own window in ascending code order.  (A second scan
// over the union of the absolute windows, chosen per wavefront when it has no more steps, was
// measured: at best 3 % faster on weights at b = 4, slower everywhere else.)
// ---------------------------------------------------------------------------------------
template <int FMT>
__device__ __forceinline__ uint32_t ceil_code(float y)      // smallest code >= 1 with value >= y
{
    uint32_t c = sf_encode_rne<FMT>(y);
    if (sf_decode<FMT>(c) < y) c = min(c + 1u, (uint32_t)ScaleFmt<FMT>::kMaxCode);
    return max(c, 1u);
}

// Per block of the lane: the window [lo, hi] of codes that can win.
template <int B, int FMT>
__device__ __forceinline__ void prune_window(const float (&v)[8], uint32_t (&lo_k)[BruteState<B>::NBLK],
                                             uint32_t (&hi_k)[BruteState<B>::NBLK])
{
    constexpr int NBLK = BruteState<B>::NBLK;
    constexpr int LANES = (B < 8) ? 1 : B / 8;
    constexpr int EPB = (B < 8) ? B : 8;
    float amax[NBLK], y[8], S[NBLK];
    uint32_t cref[NBLK];
#pragma unroll
    for (int k = 0; k < NBLK; ++k) {
        float a = 0.0f;
#pragma unroll
        for (int i = 0; i < EPB; ++i) a = fmaxf(a, __builtin_fabsf(v[k * EPB + i]));
        amax[k] = group_max<LANES>(a);
        cref[k] = max(sf_encode_rne<FMT>(sixth_of(amax[k])), 1u);
        S[k] = sf_decode<FMT>(cref[k]);
        const Recip r = make_recip(S[k]);
#pragma unroll
        for (int i = 0; i < EPB; ++i) y[k * EPB + i] = quot(v[k * EPB + i], r);
    }
    const uint32_t packed = e2m1_pack8(y, 1.0f);
    float q[8], sq[8], U[4];
    e2m1_unpack8(packed, 1.0f, q);
#pragma unroll
    for (int j = 0; j < 8; ++j) { const float e = __builtin_fmaf(-q[j], S[j / EPB], v[j]); sq[j] = e * e; }
    const float p0 = sq[0] + sq[1], p1 = sq[2] + sq[3], p2 = sq[4] + sq[5], p3 = sq[6] + sq[7];
    if constexpr (B == 2) { U[0] = p0; U[1] = p1; U[2] = p2; U[3] = p3; }
    else if constexpr (B == 4) { U[0] = p0 + p1; U[1] = p2 + p3; }
    else U[0] = group_sum<B / 8>((p0 + p1) + (p2 + p3));

    // (hi2): first binade above the reference binade whose lowest scale S0 = 2^(ef - bias) already
    // loses.  thr = S0 / 4; the sum uses the tree of the block SSE.
    constexpr int kMaxUp = 5;                                            // (hi) ends the window at five or six anyway
    constexpr uint32_t kNone = 1u << 20;
    uint32_t dz[NBLK];
#pragma unroll
    for (int k = 0; k < NBLK; ++k) dz[k] = kNone;
    float vsq[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) vsq[j] = v[j] * v[j];
    // Only the widest window of a wavefront costs steps, so the search is for the first binade d at
    // which EVERY block of the wavefront loses (a block is given the lowest tested d at which it
    // loses: never too low).  With 32 blocks per wavefront that is two or three binades up and the
    // tests simply ascend from 2; with 128 or more (b <= 4) it is usually four or five, so d = 4 is
    // probed first, then 5 if some block survives it, else 3 and 2 as long as all blocks lose.
    int d = (B <= 4) ? 4 : 2;
    bool descending = false;
#pragma unroll 1
    for (int it = 0; it < 4; ++it) {                                     // uniform
        float thr[NBLK], zs[8], Z[4];
#pragma unroll
        for (int k = 0; k < NBLK; ++k)
            thr[k] = u2f(((cref[k] >> 3) + (uint32_t)(d + 127 - ScaleFmt<FMT>::kBias - 2)) << 23);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float half = 2.0f * thr[j / EPB];                      // S0 / 2
            const float gap = half - __builtin_fabsf(v[j]);
            zs[j] = (gap > 0.0f) ? fminf(vsq[j], gap * gap) : 0.0f;     // |v| < S0/4: the minimum is v^2
        }
        const float z0 = zs[0] + zs[1], z1 = zs[2] + zs[3], z2 = zs[4] + zs[5], z3 = zs[6] + zs[7];
        if constexpr (B == 2) { Z[0] = z0; Z[1] = z1; Z[2] = z2; Z[3] = z3; }
        else if constexpr (B == 4) { Z[0] = z0 + z1; Z[1] = z2 + z3; }
        else Z[0] = group_sum<B / 8>((z0 + z1) + (z2 + z3));
        bool survives = false;
#pragma unroll
        for (int k = 0; k < NBLK; ++k) {
            if (Z[k] > U[k]) dz[k] = min(dz[k], (uint32_t)d);
            else survives = true;
        }
        const bool all_lose = __builtin_amdgcn_ballot_w64(survives) == 0ull;
        if constexpr (B <= 4) {
            if (it == 0) descending = all_lose;
            if (descending) { if (!all_lose || d == 2) break; --d; }
            else { if (all_lose || d == kMaxUp) break; ++d; }
        } else {
            if (all_lose || d == kMaxUp) break;
            ++d;
        }
    }

    // (lo) at the granularity the scan has anyway: the highest code of a binade saturates least, so
    // a binade whose highest code loses is lost as a whole, with everything below it.  Nearly every
    // block settles in the first or second binade below its reference; the bisection over the
    // codes runs only if some block of the wavefront has not settled after three.
    uint32_t lo_b[NBLK];
    bool unsettled = false;
#pragma unroll
    for (int k = 0; k < NBLK; ++k) {
        const uint32_t er = cref[k] >> 3;
        lo_b[k] = kNone;
#pragma unroll
        for (int t = 1; t <= 3; ++t) {
            // highest code of binade er - t: 1.875 * 2^(er - t - bias); the sub-normal "binade" 0
            // ends with 0.875 * 2^(1 - bias)
            const int ef = (int)er - t;
            const float top_scale = (ef >= 1) ? 1.875f * u2f((uint32_t)(ef + 127 - ScaleFmt<FMT>::kBias) << 23)
                                              : 0.875f * u2f((uint32_t)(1 + 127 - ScaleFmt<FMT>::kBias) << 23);
            const float lim = 6.0f * top_scale;
            const float dd = amax[k] - lim;
            const bool loser = ef < 0 || ((lim < amax[k]) && (dd * dd > U[k]));
            if (lo_b[k] == kNone && loser) lo_b[k] = (uint32_t)max(ef + 1, 0) << 3;
        }
        unsettled |= lo_b[k] == kNone;
    }
    const bool bisect = __builtin_amdgcn_ballot_w64(unsettled) != 0ull;  // uniform

#pragma unroll
    for (int k = 0; k < NBLK; ++k) {
        uint32_t lo = 1u, hi = cref[k];                 // the bound at cref is <= U: not a loser
        if (bisect) {
#pragma unroll 1
            for (int it = 0; it < 8; ++it) {
                if (lo < hi) {
                    const uint32_t mid = (lo + hi) >> 1;
                    const float lim = 6.0f * sf_decode<FMT>(mid);
                    const float d = amax[k] - lim;
                    const bool loser = (lim < amax[k]) && (d * d > U[k]);
                    if (loser) lo = mid + 1u; else hi = mid;
                }
            }
        } else {
            lo = max(lo_b[k], 1u);
        }
        lo_k[k] = lo;
        hi_k[k] = ceil_code<FMT>(4.0f * amax[k]);
        if (dz[k] != kNone) hi_k[k] = min(hi_k[k], (((cref[k] >> 3) + dz[k]) << 3) - 1u);
    }
}

// One candidate of the relative scan: mantissa MI (uniform), power of two per block.
template <int B, int MI, int POS, class G>
__device__ __forceinline__ void try_candidate_rel(const float (&v)[8], const float (&w)[8],
                                                  const float (&scale2)[BruteState<B>::NBLK], G& g)
{
    constexpr int EPB = (B < 8) ? B : 8;
    const uint32_t packed = e2m1_pack8_scales<EPB>(w, scale2);
    float q2[8], sq[8];
    e2m1_unpack2<0>(packed, scale2[0 / EPB], q2[0], q2[1]);
    e2m1_unpack2<1>(packed, scale2[2 / EPB], q2[2], q2[3]);
    e2m1_unpack2<2>(packed, scale2[4 / EPB], q2[4], q2[5]);
    e2m1_unpack2<3>(packed, scale2[6 / EPB], q2[6], q2[7]);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        float e;
        if constexpr (MI == 0) e = v[j] - q2[j];
        else e = __builtin_fmaf(-q2[j], mant_value(MI), v[j]);
        sq[j] = e * e;
    }
    const float p0 = sq[0] + sq[1], p1 = sq[2] + sq[3], p2 = sq[4] + sq[5], p3 = sq[6] + sq[7];
    if constexpr (B == 2) {
        g.template put<POS>(0, p0); g.template put<POS>(1, p1);
        g.template put<POS>(2, p2); g.template put<POS>(3, p3);
    } else if constexpr (B == 4) {
        g.template put<POS>(0, p0 + p1); g.template put<POS>(1, p2 + p3);
    } else {
        g.template put<POS>(0, group_sum<B / 8>((p0 + p1) + (p2 + p3)));
    }
    __builtin_amdgcn_sched_barrier(0);
}

template <int B, int MI, class G>
__device__ __forceinline__ void try_binade_rel_from(const float (&v)[8], const float (&w)[8][8],
                                                    const float (&scale2)[BruteState<B>::NBLK], G& g)
{
    if constexpr (MI < 8) {
        try_candidate_rel<B, MI, MI>(v, w[MI], scale2, g);
        try_binade_rel_from<B, MI + 1>(v, w, scale2, g);
    }
}

// Value of a power-of-two scale byte (0 .. 254); 2^-127 is a sub-normal float.
__device__ __forceinline__ float pow2_scale(uint32_t code)
{
    return (code == 0u) ? u2f(0x00400000u) : u2f(code << 23);
}

// The 8 codes code0 .. code0 + 7 of the power-of-two format; code 255 is not a number.
template <int B, int POS, class G>
__device__ __forceinline__ void try_pow2_from(const float (&v)[8], uint32_t code0, G& g)
{
    if constexpr (POS < 8) {
        if (POS < 7 || code0 + 7u <= 254u) try_candidate<B, 0, POS>(v, v, pow2_scale(code0 + POS), g);
        try_pow2_from<B, POS + 1>(v, code0, g);
    }
}

// Search for the lane's 8 values (already divided by T): winner codes, packed nibbles, SSE.
template <int B, int FMT, bool PRUNE>
__device__ __forceinline__ void brute_search(const float (&v)[8], uint32_t& packed, BruteState<B>& st)
{
    constexpr int NBLK = BruteState<B>::NBLK;
    constexpr int EPB = (B < 8) ? B : 8;
    constexpr int bias = ScaleFmt<FMT>::kBias;
    constexpr int emin = 1 - bias;                                      // exponent of the first binade

    constexpr uint32_t lo_w = 1u, hi_w = (uint32_t)ScaleFmt<FMT>::kMaxCode;
    static_assert(!PRUNE, "the pruned search is brute_search_pruned");

    float w[8][8];
#pragma unroll
    for (int j = 0; j < 8; ++j) w[0][j] = v[j];
#pragma unroll
    for (int i = 1; i < 8; ++i) {
#pragma unroll
        for (int j = 0; j < 8; ++j) w[i][j] = quot(v[j], Recip{mant_rhi(i), mant_rlo(i)});
    }
#pragma unroll
    for (int k = 0; k < NBLK; ++k) { st.best_sse[k] = __builtin_inff(); st.best_code[k] = 1u; }

    // sub-normal codes 1..7 = j * 2^(emin-3): 1, 2, 3 = 1.5*2, 4, 5 = 1.25*4, 6 = 1.5*4, 7 = 1.75*4
    const float s1 = u2f((uint32_t)(127 + emin - 3) << 23);
    const float s2 = u2f((uint32_t)(127 + emin - 2) << 23);
    const float s4 = u2f((uint32_t)(127 + emin - 1) << 23);
    if (lo_w < 8u) {                                                    // uniform
        GroupArgMin<B> g;
        g.begin();
        try_candidate<B, 0, 0>(v, w[0], s1, g);
        try_candidate<B, 0, 1>(v, w[0], s2, g);
        try_candidate<B, 4, 2>(v, w[4], s2, g);
        try_candidate<B, 0, 3>(v, w[0], s4, g);
        try_candidate<B, 2, 4>(v, w[2], s4, g);
        try_candidate<B, 4, 5>(v, w[4], s4, g);
        try_candidate<B, 6, 6>(v, w[6], s4, g);
        g.end(st, 1u);
    }

    // normal codes: exponent field ef = 1 .. kMaxCode >> 3, value (1 + mi/8) * 2^(ef - bias)
    for (uint32_t ef = max(lo_w >> 3, 1u); ef <= (hi_w >> 3); ++ef) {
        const float scale2 = u2f((ef + (uint32_t)(127 - bias)) << 23);
        try_binade<B, FMT>(v, w, scale2, ef << 3, st);
    }

    // codes of the winners
    float y[8];
#pragma unroll
    for (int k = 0; k < NBLK; ++k) {
        const Recip r = make_recip(sf_decode<FMT>(st.best_code[k]));
#pragma unroll
        for (int i = 0; i < EPB; ++i) y[k * EPB + i] = quot(v[k * EPB + i], r);
    }
    packed = e2m1_pack8(y, 1.0f);
}

// Pruned search: windows, then the relative scan described above.
template <int B, int FMT>
__device__ __forceinline__ void brute_search_pruned(const float (&v)[8], uint32_t& packed, BruteState<B>& st)
{
    constexpr int NBLK = BruteState<B>::NBLK;
    constexpr int EPB = (B < 8) ? B : 8;
    constexpr int bias = ScaleFmt<FMT>::kBias;
    constexpr int emin = 1 - bias;
    constexpr int top = ScaleFmt<FMT>::kMaxCode >> 3;                   // last binade; its position 7 is not a number

    uint32_t lo_k[NBLK], hi_k[NBLK];
    prune_window<B, FMT>(v, lo_k, hi_k);
    // Steps of the scan: every block starts at the first binade of its OWN window, so the
    // wavefront needs as many steps as its widest window has binades.
    int w_max = -1;
    bool sub = false;
#pragma unroll
    for (int k = 0; k < NBLK; ++k) {
        w_max = max(w_max, (int)(hi_k[k] >> 3) - max((int)(lo_k[k] >> 3), 1));
        sub |= lo_k[k] < 8u;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) w_max = max(w_max, __shfl_xor(w_max, off, 64));
    w_max = __builtin_amdgcn_readfirstlane(w_max);
    const bool any_sub = __builtin_amdgcn_ballot_w64(sub) != 0ull;

    float w[8][8];
#pragma unroll
    for (int j = 0; j < 8; ++j) w[0][j] = v[j];
#pragma unroll
    for (int i = 1; i < 8; ++i) {
#pragma unroll
        for (int j = 0; j < 8; ++j) w[i][j] = quot(v[j], Recip{mant_rhi(i), mant_rlo(i)});
    }
#pragma unroll
    for (int k = 0; k < NBLK; ++k) { st.best_sse[k] = __builtin_inff(); st.best_code[k] = 1u; }

    if (any_sub) {                                                      // uniform: codes 1 .. 7
        const float s1 = u2f((uint32_t)(127 + emin - 3) << 23);
        const float s2 = u2f((uint32_t)(127 + emin - 2) << 23);
        const float s4 = u2f((uint32_t)(127 + emin - 1) << 23);
        GroupArgMin<B> g;
        g.begin();
        try_candidate<B, 0, 0>(v, w[0], s1, g);
        try_candidate<B, 0, 1>(v, w[0], s2, g);
        try_candidate<B, 4, 2>(v, w[4], s2, g);
        try_candidate<B, 0, 3>(v, w[0], s4, g);
        try_candidate<B, 2, 4>(v, w[2], s4, g);
        try_candidate<B, 4, 5>(v, w[4], s4, g);
        try_candidate<B, 6, 6>(v, w[6], s4, g);
        g.end(st, 1u);
    }

    for (int t = 0; t <= w_max; ++t) {                                  // uniform
        float scale2[NBLK];
        uint32_t code0[NBLK];
        bool ok[NBLK], last[NBLK];
#pragma unroll
        for (int k = 0; k < NBLK; ++k) {
            const int ef = max((int)(lo_k[k] >> 3), 1) + t;             // this block's binade in step t
            ok[k] = ef <= (int)(hi_k[k] >> 3);
            const int efc = min(ef, top);
            last[k] = efc == top;
            scale2[k] = u2f((uint32_t)(efc + 127 - bias) << 23);
            code0[k] = (uint32_t)efc << 3;
        }
        GroupArgMin<B> g;
        g.begin();
        try_binade_rel_from<B, 0>(v, w, scale2, g);
#pragma unroll
        for (int k = 0; k < NBLK; ++k) g.drop_last(k, last[k]);
        g.end(st, code0, ok);
    }

    // codes of the winners
    float y[8];
#pragma unroll
    for (int k = 0; k < NBLK; ++k) {
        const Recip r = make_recip(sf_decode<FMT>(st.best_code[k]));
#pragma unroll
        for (int i = 0; i < EPB; ++i) y[k * EPB + i] = quot(v[k * EPB + i], r);
    }
    packed = e2m1_pack8(y, 1.0f);
}

// The same over the 255 power-of-two scales (bytes 0x00 .. 0xFE): no quotient, the conversion
// applies 2^k itself, for the candidates and for the winners' codes.
template <int B>
__device__ __forceinline__ void brute_search_pow2(const float (&v)[8], uint32_t& packed, BruteState<B>& st)
{
    constexpr int NBLK = BruteState<B>::NBLK;
    constexpr int EPB = (B < 8) ? B : 8;
#pragma unroll
    for (int k = 0; k < NBLK; ++k) { st.best_sse[k] = __builtin_inff(); st.best_code[k] = 0u; }
    for (uint32_t code0 = 0u; code0 < 256u; code0 += 8u) {
        GroupArgMin<B> g;
        g.begin();
        try_pow2_from<B, 0>(v, code0, g);
        g.end(st, code0);
    }
    float S[NBLK];
#pragma unroll
    for (int k = 0; k < NBLK; ++k) S[k] = pow2_scale(st.best_code[k]);
    packed = e2m1_pack8_scales<EPB>(v, S);
}

// Scale value of a winner byte.
template <int FMT>
__device__ __forceinline__ float brute_scale_value(uint32_t code)
{
    if constexpr (FMT == kE8M0) return pow2_scale(code);
    else return sf_decode<FMT>(code);
}

// Clipping-only part of the winners' block SSE (appendix figure "Clipping only MSE"): elements with
// |v| > 6 S quantise to +-6; their squared residuals, summed by the tree of the block SSE.
template <int B>
__device__ __forceinline__ void brute_clip_sse(const float (&v)[8], const float (&S)[BruteState<B>::NBLK], float (&clip)[4])
{
    constexpr int EPB = (B < 8) ? B : 8;
    float sq[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float s = S[j / EPB];
        const float q = u2f(0x40C00000u | (f2u(v[j]) & 0x80000000u));          // +-6
        const float e = __builtin_fmaf(-q, s, v[j]);
        sq[j] = (__builtin_fabsf(v[j]) > 6.0f * s) ? e * e : 0.0f;
    }
    const float p0 = sq[0] + sq[1], p1 = sq[2] + sq[3], p2 = sq[4] + sq[5], p3 = sq[6] + sq[7];
    if constexpr (B == 2) { clip[0] = p0; clip[1] = p1; clip[2] = p2; clip[3] = p3; }
    else if constexpr (B == 4) { clip[0] = p0 + p1; clip[1] = p2 + p3; }
    else clip[0] = group_sum<B / 8>((p0 + p1) + (p2 + p3));
}

template <int DT, int B, int FMT, bool HAS_T, bool PRUNE>
__global__ void __launch_bounds__(kThreads)
brute_kernel(const void* __restrict__ x, int64_t n_full, float T_arg,
             const float* __restrict__ absmax_dev, float* __restrict__ t_out,
             uint32_t* __restrict__ codes, uint8_t* __restrict__ scales, float* __restrict__ sse_out,
             float* __restrict__ clip_out)
{
    constexpr int NBLK = BruteState<B>::NBLK;
    constexpr int LANES = (B < 8) ? 1 : B / 8;
    float T = T_arg;
    if constexpr (HAS_T) {
        if (absmax_dev) {                                            // T from the abs-max in device memory
            T = tensor_scale_of<FMT>(*absmax_dev);
            if (t_out && blockIdx.x == 0 && threadIdx.x == 0) *t_out = T;
        }
    }

    const int64_t stride = (int64_t)gridDim.x * kThreads;
    int64_t chunk = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    int64_t base = chunk - (threadIdx.x & 63);

    for (; base < n_full; base += stride, chunk += stride) {
        float v[8];
        if (chunk < n_full) load8<DT>(x, chunk << 3, v);
        else {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = 0.0f;
        }
        if constexpr (HAS_T) {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = v[i] / T;
        }
        uint32_t packed;
        BruteState<B> st;
        if constexpr (FMT == kE8M0) brute_search_pow2<B>(v, packed, st);
        else if constexpr (PRUNE) brute_search_pruned<B, FMT>(v, packed, st);
        else brute_search<B, FMT, false>(v, packed, st);
        float clip[4];
        if (clip_out) {                                                 // uniform
            float S_best[NBLK];
#pragma unroll
            for (int k = 0; k < NBLK; ++k) S_best[k] = brute_scale_value<FMT>(st.best_code[k]);
            brute_clip_sse<B>(v, S_best, clip);
        }

        if (chunk < n_full) {
            codes[chunk] = packed;
            if constexpr (B >= 8) {
                if ((threadIdx.x & (LANES - 1)) == 0) {
                    const int64_t blk = chunk / LANES;
                    scales[blk] = (uint8_t)st.best_code[0];
                    if (sse_out) sse_out[blk] = st.best_sse[0];
                    if (clip_out) clip_out[blk] = clip[0];
                }
            } else {
                const int64_t blk0 = chunk * NBLK;
#pragma unroll
                for (int k = 0; k < NBLK; ++k) {
                    scales[blk0 + k] = (uint8_t)st.best_code[k];
                    if (sse_out) sse_out[blk0 + k] = st.best_sse[k];
                    if (clip_out) clip_out[blk0 + k] = clip[k];
                }
            }
        }
    }
}

// Ragged tail (n not a multiple of 8; b = 2 or 4 only): lane 0 of one wavefront.
template <int DT, int B, int FMT, bool HAS_T, bool PRUNE>
__global__ void __launch_bounds__(64)
brute_tail_kernel(const void* __restrict__ x, int64_t first, int count, float T_arg,
                  const float* __restrict__ absmax_dev, float* __restrict__ t_out,
                  uint8_t* __restrict__ codes, uint8_t* __restrict__ scales, float* __restrict__ sse_out,
                  float* __restrict__ clip_out)
{
    constexpr int NBLK = BruteState<B>::NBLK;
    float T = T_arg;
    if constexpr (HAS_T) {
        if (absmax_dev) {
            T = tensor_scale_of<FMT>(*absmax_dev);
            if (t_out && threadIdx.x == 0) *t_out = T;      // t_out is passed only when no main kernel runs
        }
    }
    float v[8];
    load_partial<DT>(x, first, (threadIdx.x == 0) ? count : 0, v);
    if constexpr (HAS_T) {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = v[i] / T;
    }
    uint32_t packed;
    BruteState<B> st;
    if constexpr (FMT == kE8M0) brute_search_pow2<B>(v, packed, st);
    else if constexpr (PRUNE) brute_search_pruned<B, FMT>(v, packed, st);
    else brute_search<B, FMT, false>(v, packed, st);
    float S_best[NBLK], clip[4];
    for (int k = 0; k < NBLK; ++k) S_best[k] = brute_scale_value<FMT>(st.best_code[k]);
    brute_clip_sse<B>(v, S_best, clip);
    if (threadIdx.x != 0) return;
    for (int i = 0; i < count / 2; ++i) codes[first / 2 + i] = (uint8_t)(packed >> (8 * i));
    for (int k = 0; k < NBLK; ++k) {
        if (k < count / B) {
            scales[first / B + k] = (uint8_t)st.best_code[k];
            if (sse_out) sse_out[first / B + k] = st.best_sse[k];
            if (clip_out) clip_out[first / B + k] = clip[k];
        }
    }
}

template <int DT, int B, int FMT, bool PRUNE>
static hipError_t launch_f(const StreamArgs& a)
{
    const int64_t n_full = a.n / 8;
    const int count = (int)(a.n - n_full * 8);
    const bool has_t = (a.absmax_dev != nullptr) || (a.T != 1.0f);
    if (n_full > 0) {
        const int64_t need = (n_full + kThreads - 1) / kThreads;
        const dim3 grid((unsigned)(need < 256 * 8 ? need : 256 * 8)), block(kThreads);
        if (has_t)
            hipLaunchKernelGGL((brute_kernel<DT, B, FMT, true, PRUNE>), grid, block, 0, a.stream,
                               a.x, n_full, a.T, a.absmax_dev, a.t_out, (uint32_t*)a.codes, a.scales, a.sse, a.clip);
        else
            hipLaunchKernelGGL((brute_kernel<DT, B, FMT, false, PRUNE>), grid, block, 0, a.stream,
                               a.x, n_full, a.T, a.absmax_dev, a.t_out, (uint32_t*)a.codes, a.scales, a.sse, a.clip);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if constexpr (B < 8) {
        if (count > 0) {
            float* t_out_tail = (n_full > 0) ? nullptr : a.t_out;
            if (has_t)
                hipLaunchKernelGGL((brute_tail_kernel<DT, B, FMT, true, PRUNE>), dim3(1), dim3(64), 0, a.stream,
                                   a.x, n_full * 8, count, a.T, a.absmax_dev, t_out_tail, a.codes, a.scales, a.sse, a.clip);
            else
                hipLaunchKernelGGL((brute_tail_kernel<DT, B, FMT, false, PRUNE>), dim3(1), dim3(64), 0, a.stream,
                                   a.x, n_full * 8, count, a.T, a.absmax_dev, t_out_tail, a.codes, a.scales, a.sse, a.clip);
        }
    }
    return hipGetLastError();
}

template <int DT, int B>
static hipError_t launch_b(const StreamArgs& a)
{
    const bool prune = (a.recipe == 5);
    if (a.scale_fmt == kE8M0) return launch_f<DT, B, kE8M0, false>(a);          // the host refuses the pruned form
    if (a.scale_fmt == kE4M3) return prune ? launch_f<DT, B, kE4M3, true>(a) : launch_f<DT, B, kE4M3, false>(a);
    return prune ? launch_f<DT, B, kUE5M3, true>(a) : launch_f<DT, B, kUE5M3, false>(a);
}

template <int DT>
static hipError_t launch_d(const StreamArgs& a)
{
    switch (a.block) {
        case 2: return launch_b<DT, 2>(a);
        case 4: return launch_b<DT, 4>(a);
        case 8: return launch_b<DT, 8>(a);
        case 16: return launch_b<DT, 16>(a);
        case 32: return launch_b<DT, 32>(a);
        case 64: return launch_b<DT, 64>(a);
        default: return launch_b<DT, 128>(a);
    }
}

hipError_t launch_brute(const StreamArgs& a)
{
    return (a.dtype == kBF16) ? launch_d<kBF16>(a) : launch_d<kF32>(a);
}

}  // namespace mxq
