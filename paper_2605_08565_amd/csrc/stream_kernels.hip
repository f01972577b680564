// Streaming recipes of Section 2: abs-max scale (Eq. 2; Eq. 1 for power-of-two scales),
// prevent-zero clamp (Eq. 3) and 4-over-6 (Eq. 4), one pass over the tensor.
//
// Mapping: every lane owns 8 consecutive elements (one 128-bit load for bf16, two for fp32),
// so a block of b >= 8 elements is b/8 neighbouring lanes of one DPP row and a block of
// b < 8 sits inside a lane.  Per lane the kernel emits one dword of packed codes; the first
// lane of a block emits the scale byte and the block SSE.  The next chunk's load is issued
// before the current chunk is processed.  HBM-bound by design: algorithmic traffic is
// sizeof(in) + 0.5 + 5/b bytes per element.
#include "mxq_device.hpp"
#include "mxq_launch.hpp"

#ifndef MXQ_STREAM_ITEMS
#define MXQ_STREAM_ITEMS 1
#endif

namespace mxq {

// Eq. 2 / Eq. 3: scale codes from the block abs-max for M = 6 and (4-over-6 only) M = 4.
// `floor_code` is 1 under prevent-zero (eps_SF is code 1 in both formats), else 0.  For E4M3 one
// v_cvt_pk_fp8_f32 rounds both quotients.
template <int FMT, bool FOUR6>
__device__ __forceinline__ void absmax_codes(float amax, uint32_t floor_code, uint32_t& c6, uint32_t& c4)
{
    const float y6 = sixth_of(amax);
    const float y4 = quarter_of(amax);
    if constexpr (FMT == kE4M3) {
        const float m = ScaleFmt<kE4M3>::kMaxValue;
        int old;                                       // the conversion writes the low half; the high half is never read
        asm volatile("" : "=v"(old));
        const uint32_t both = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(fminf(y6, m), fminf(y4, m), old, false);
        c6 = max(both & 0xFFu, floor_code);
        c4 = FOUR6 ? max((both >> 8) & 0xFFu, floor_code) : 0u;
    } else {
        c6 = max(sf_encode_rne<FMT>(y6), floor_code);
        c4 = FOUR6 ? max(sf_encode_rne<FMT>(y4), floor_code) : 0u;
    }
}

// Quantise the lane's 8 values (NBLK blocks of EPB elements, one scale code each) under
// table scales: packed nibbles and the 8 squared residuals.
template <int NBLK, int EPB>
__device__ __forceinline__ void quant_lane(const float (&v)[8], const uint32_t (&code)[NBLK],
                                           const ScaleEntry* tab, uint32_t& packed, float (&sq)[8], float (&S)[NBLK])
{
    float y[8];
#pragma unroll
    for (int k = 0; k < NBLK; ++k) {
        const ScaleEntry se = tab[code[k]];
        S[k] = se.S;
#pragma unroll
        for (int i = 0; i < EPB; ++i) {
            const int j = k * EPB + i;
            y[j] = quot(v[j], Recip{se.rhi, se.rlo});
        }
    }
    packed = e2m1_pack8(y, 1.0f);
    float q[8];
    e2m1_unpack8(packed, 1.0f, q);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float e = __builtin_fmaf(-q[j], S[j / EPB], v[j]);   // q*S is exact: one rounding
        sq[j] = e * e;
    }
}

// Same under power-of-two scales 2^(code-127): v / 2^k is exact, so the conversion
// instruction applies each block's scale itself and the inverse conversion returns q * S.
template <int NBLK, int EPB>
__device__ __forceinline__ void quant_lane_pow2(const float (&v)[8], const uint32_t (&code)[NBLK],
                                                uint32_t& packed, float (&sq)[8], float (&S)[NBLK])
{
#pragma unroll
    for (int k = 0; k < NBLK; ++k) S[k] = (code[k] == 0u) ? u2f(0x00400000u) : u2f(code[k] << 23);
    packed = e2m1_pack8_scales<EPB>(v, S);
    float qS[8];
    e2m1_unpack2<0>(packed, S[0 / EPB], qS[0], qS[1]);
    e2m1_unpack2<1>(packed, S[2 / EPB], qS[2], qS[3]);
    e2m1_unpack2<2>(packed, S[4 / EPB], qS[4], qS[5]);
    e2m1_unpack2<3>(packed, S[6 / EPB], qS[6], qS[7]);
#pragma unroll
    for (int j = 0; j < 8; ++j) { const float e = v[j] - qS[j]; sq[j] = e * e; }
}

// Block SSE: balanced tree in index order, inside the lane and then across the block's lanes.
// For b < 8 the lane holds 8/b blocks; their sums come back in sse[0 .. 8/b).
template <int B>
__device__ __forceinline__ void block_sse(const float (&sq)[8], float (&sse)[4])
{
    const float p0 = sq[0] + sq[1], p1 = sq[2] + sq[3], p2 = sq[4] + sq[5], p3 = sq[6] + sq[7];
    if constexpr (B == 2) {
        sse[0] = p0; sse[1] = p1; sse[2] = p2; sse[3] = p3;
    } else if constexpr (B == 4) {
        sse[0] = p0 + p1; sse[1] = p2 + p3;
    } else {
        sse[0] = group_sum<B / 8>((p0 + p1) + (p2 + p3));
    }
}

// Clipping-only part of the block SSE (appendix figure "Clipping only MSE"): the squared residuals
// of the elements that saturate, |v| > 6 S (the same decision as fl32(|v| / S) > 6, because 6 S is
// exact), others contribute +0; S = 0 clips nothing.  A saturating element quantises to +-6, so its
// squared residual is the one the block SSE already holds.
template <int B, int NBLK, int EPB>
__device__ __forceinline__ void block_clip_sse(const float (&v)[8], const float (&sq)[8], const float (&S)[NBLK],
                                               float (&clip)[4])
{
    float csq[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float s = S[j / EPB];
        csq[j] = (__builtin_fabsf(v[j]) > 6.0f * s && s > 0.0f) ? sq[j] : 0.0f;
    }
    block_sse<B>(csq, clip);
}

// Division by the per-tensor scale T of hierarchical scaling: div_by_T (reciprocal + one FMA
// refinement, exact inside the range fast_division_ok / fast_division_unsafe_amax delimit) or the
// plain IEEE division.
enum : int { kNoT = 0, kFastT = 1, kSlowT = 2, kDynT = 3 };   // kDynT: T comes from device memory, one of
                                                              // the other three is chosen at run time

template <int NBLK, int EPB, int LANES>
__device__ __forceinline__ void block_amax(const float (&v)[8], float (&amax)[NBLK])
{
#pragma unroll
    for (int k = 0; k < NBLK; ++k) {
        float a = 0.0f;
#pragma unroll
        for (int i = 0; i < EPB; ++i) a = fmaxf(a, __builtin_fabsf(v[k * EPB + i]));
        amax[k] = group_max<LANES>(a);
    }
}

// Division by the per-tensor scale (MODE: none / reciprocal-refined / plain) and the block
// abs-max of the adjusted values.
template <int MODE, int NBLK, int EPB, int LANES>
__device__ __forceinline__ void adjust_and_amax(float (&v)[8], float T, float rT, float (&amax)[NBLK])
{
    if constexpr (MODE == kSlowT) {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = v[i] / T;            // IEEE division
        block_amax<NBLK, EPB, LANES>(v, amax);
    } else if constexpr (MODE == kFastT) {
        float raw[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) { raw[i] = v[i]; v[i] = div_by_T(raw[i], T, rT); }
        block_amax<NBLK, EPB, LANES>(v, amax);
        bool unsafe = false;
#pragma unroll
        for (int k = 0; k < NBLK; ++k)                  // 0 < amax < 2^-40  or  amax > 2^90
            unsafe |= fast_division_unsafe_amax(amax[k]);
        if (__builtin_amdgcn_ballot_w64(unsafe) != 0ull) {       // rare, wave-uniform
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = raw[i] / T;
            block_amax<NBLK, EPB, LANES>(v, amax);
        }
    } else {
        block_amax<NBLK, EPB, LANES>(v, amax);
    }
}

// Everything between the load and the store for one lane's 8 values.  `tdyn` (one of kNoT,
// kFastT, kSlowT; wave-uniform) is read only when TMODE == kDynT.
template <int B, int FMT, bool FOUR6, int TMODE, bool CLIP>
__device__ __forceinline__ void process_chunk(float (&v)[8], float T, float rT, int tdyn, bool pz,
                                              const ScaleEntry* tab, uint32_t& packed,
                                              uint32_t (&code_out)[(B < 8) ? 8 / B : 1], float (&sse_sel)[4],
                                              float (&clip_sel)[4])
{
    constexpr int NBLK = (B < 8) ? 8 / B : 1;          // blocks inside one lane
    constexpr int LANES = (B < 8) ? 1 : B / 8;         // lanes per block
    constexpr int EPB = (B < 8) ? B : 8;               // elements of one block inside a lane

    float amax[NBLK];
    if constexpr (TMODE == kDynT) {
        if (tdyn == kNoT) adjust_and_amax<kNoT, NBLK, EPB, LANES>(v, T, rT, amax);
        else if (tdyn == kFastT) adjust_and_amax<kFastT, NBLK, EPB, LANES>(v, T, rT, amax);
        else adjust_and_amax<kSlowT, NBLK, EPB, LANES>(v, T, rT, amax);
    } else {
        adjust_and_amax<TMODE, NBLK, EPB, LANES>(v, T, rT, amax);
    }

    float sq[8], S[NBLK];
    if constexpr (FMT == kE8M0) {
#pragma unroll
        for (int k = 0; k < NBLK; ++k) code_out[k] = pow2_code(amax[k]);
        quant_lane_pow2<NBLK, EPB>(v, code_out, packed, sq, S);
        block_sse<B>(sq, sse_sel);
        if constexpr (CLIP) block_clip_sse<B, NBLK, EPB>(v, sq, S, clip_sel);
    } else {
        uint32_t c4[NBLK];
        const uint32_t floor_code = pz ? 1u : 0u;
#pragma unroll
        for (int k = 0; k < NBLK; ++k) absmax_codes<FMT, FOUR6>(amax[k], floor_code, code_out[k], c4[k]);
        quant_lane<NBLK, EPB>(v, code_out, tab, packed, sq, S);
        block_sse<B>(sq, sse_sel);
        if constexpr (CLIP) block_clip_sse<B, NBLK, EPB>(v, sq, S, clip_sel);
        if constexpr (FOUR6) {
            uint32_t packed4;
            float sse4[4], clip4[4];
            quant_lane<NBLK, EPB>(v, c4, tab, packed4, sq, S);
            block_sse<B>(sq, sse4);
            if constexpr (CLIP) block_clip_sse<B, NBLK, EPB>(v, sq, S, clip4);
            // Eq. 4: M = 4 only when its SSE is strictly lower
#pragma unroll
            for (int k = 0; k < NBLK; ++k) {
                if (sse4[k] < sse_sel[k]) {
                    constexpr uint32_t m = (EPB == 8) ? 0xFFFFFFFFu : ((1u << ((4 * EPB) & 31)) - 1u);
                    const uint32_t mask = m << ((4 * EPB * k) & 31);
                    packed = (packed & ~mask) | (packed4 & mask);
                    code_out[k] = c4[k];
                    sse_sel[k] = sse4[k];
                    if constexpr (CLIP) clip_sel[k] = clip4[k];
                }
            }
        }
    }
}

template <int DT> struct RawChunk;
template <> struct RawChunk<kBF16> { u32x4 a; };
template <> struct RawChunk<kF32> { u32x4 a, b; };

// `tile` points at the workgroup's 256 chunks (wave-uniform), `tid` is the lane's chunk inside
// it and `chunks` the number of valid chunks (lanes beyond them re-read the last valid data).
// bf16: one 128-bit load per lane.  fp32: a chunk is two 128-bit vectors; so that every load
// instruction of a wavefront covers 1 KiB without gaps, lane l of wave w reads vectors
// 128w + l and 128w + 64 + l, and widen() below hands every lane its own chunk through LDS.
template <int DT>
__device__ __forceinline__ RawChunk<DT> load_raw(const u32x4* __restrict__ tile, uint32_t tid, uint32_t chunks)
{
    RawChunk<DT> r;
    if constexpr (DT == kBF16) {
        r.a = __builtin_nontemporal_load(tile + min(tid, chunks - 1u));
    } else {
        const uint32_t j = 2u * (tid & ~63u) + (tid & 63u);
        const uint32_t last = 2u * chunks - 1u;
        r.a = __builtin_nontemporal_load(tile + min(j, last));
        r.b = __builtin_nontemporal_load(tile + min(j + 64u, last));
    }
    return r;
}

// Raw registers -> the lane's 8 consecutive elements as fp32.  fp32 input: the wavefront
// writes its two 1 KiB load results to its private 2 KiB of LDS and every lane reads back
// vectors 2l and 2l + 1.  LDS operations of one wavefront execute in program order, so no
// barrier instruction is needed; the fences keep the compiler from reordering across them.
template <int DT>
__device__ __forceinline__ void widen(const RawChunk<DT>& r, float (&v)[8], u32x4* wave_lds)
{
    if constexpr (DT == kBF16) {
        v[0] = u2f(r.a.x << 16); v[1] = u2f(r.a.x & 0xFFFF0000u);
        v[2] = u2f(r.a.y << 16); v[3] = u2f(r.a.y & 0xFFFF0000u);
        v[4] = u2f(r.a.z << 16); v[5] = u2f(r.a.z & 0xFFFF0000u);
        v[6] = u2f(r.a.w << 16); v[7] = u2f(r.a.w & 0xFFFF0000u);
    } else {
        const uint32_t l = threadIdx.x & 63u;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        wave_lds[l] = r.a;
        wave_lds[64u + l] = r.b;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        const u32x4 a = wave_lds[2u * l], b = wave_lds[2u * l + 1u];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        v[0] = u2f(a.x); v[1] = u2f(a.y); v[2] = u2f(a.z); v[3] = u2f(a.w);
        v[4] = u2f(b.x); v[5] = u2f(b.y); v[6] = u2f(b.z); v[7] = u2f(b.w);
    }
}

// Results of one lane for one tile, kept in registers until they are stored.
template <int B>
struct TileOut {
    static constexpr int NBLK = (B < 8) ? 8 / B : 1;
    uint32_t packed;
    uint32_t code[NBLK];
    float sse[4];
    float clip[4];       // clipping-only SSE; carried only by the kernels that output it
};

// The complete chunks are cut into slices of 256 chunks (one chunk per lane).  Slice indices
// are 32-bit and wave-uniform, so all tile arithmetic runs on the scalar unit and every address
// is a scalar base plus a 32-bit lane offset.
struct Slices {
    uint32_t count;        // number of slices
    uint32_t last;         // chunks in the last slice, 1 .. 256
    __device__ __forceinline__ uint32_t chunks(uint32_t s) const { return (s + 1u == count) ? last : (uint32_t)kThreads; }
};

// Stores of one slice.
template <int B>
__device__ __forceinline__ void store_slice(const TileOut<B>& o, uint32_t s, Slices sl,
                                            uint32_t* __restrict__ codes, uint8_t* __restrict__ scales,
                                            float* __restrict__ sse_out, float* __restrict__ clip_out)
{
    constexpr int NBLK = TileOut<B>::NBLK;
    constexpr int LANES = (B < 8) ? 1 : B / 8;
    const uint32_t tid = threadIdx.x;
    if (s >= sl.count) return;                                       // uniform
    const uint64_t c0 = (uint64_t)s * kThreads;                      // first chunk of the slice
    if (tid < sl.chunks(s)) {
        __builtin_nontemporal_store(o.packed, codes + c0 + tid);
        if constexpr (B >= 8) {
            if ((tid & (LANES - 1)) == 0) {
                const uint32_t blk = tid / LANES;
                (scales + c0 / LANES)[blk] = (uint8_t)o.code[0];
                if (sse_out) (sse_out + c0 / LANES)[blk] = o.sse[0];
                if (clip_out) (clip_out + c0 / LANES)[blk] = o.clip[0];
            }
        } else if constexpr (NBLK == 2) {
            reinterpret_cast<uint16_t*>(scales + c0 * 2)[tid] = (uint16_t)(o.code[0] | (o.code[1] << 8));
            if (sse_out) reinterpret_cast<float2*>(sse_out + c0 * 2)[tid] = make_float2(o.sse[0], o.sse[1]);
            if (clip_out) reinterpret_cast<float2*>(clip_out + c0 * 2)[tid] = make_float2(o.clip[0], o.clip[1]);
        } else {
            reinterpret_cast<uint32_t*>(scales + c0 * 4)[tid] =
                o.code[0] | (o.code[1] << 8) | (o.code[2] << 16) | (o.code[3] << 24);
            if (sse_out)
                reinterpret_cast<float4*>(sse_out + c0 * 4)[tid] =
                    make_float4(o.sse[0], o.sse[1], o.sse[2], o.sse[3]);
            if (clip_out)
                reinterpret_cast<float4*>(clip_out + c0 * 4)[tid] =
                    make_float4(o.clip[0], o.clip[1], o.clip[2], o.clip[3]);
        }
    }
}

// A workgroup tile is kItems consecutive slices; every lane owns one chunk of each slice.
constexpr int kItems = MXQ_STREAM_ITEMS;

template <int DT>
__device__ __forceinline__ void load_tile(RawChunk<DT> (&buf)[kItems], const void* __restrict__ x,
                                          uint32_t s0, Slices sl)
{
    constexpr uint64_t kVecPerChunk = (DT == kBF16) ? 1 : 2;
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const uint32_t s = s0 + (uint32_t)i;
        if (s < sl.count) {                                          // uniform
            buf[i] = load_raw<DT>(static_cast<const u32x4*>(x) + (uint64_t)s * kThreads * kVecPerChunk,
                                  (uint32_t)threadIdx.x, sl.chunks(s));
        }
    }
}

// One step of the software pipeline for the tile at slice s0 whose raw data sits in `cur`:
//   wait until `cur` has landed -> issue the stores of the PREVIOUS tile -> issue the loads of
//   the NEXT tile into `nxt` -> quantise `cur` into `out`.
// On gfx9 loads and stores share one in-order counter, so the wait at the top covers every
// memory operation still in flight; with this order all of them were issued a whole compute
// phase earlier and the wait is short.
template <int DT, int B, int FMT, bool FOUR6, int TMODE, bool CLIP>
__device__ __forceinline__ void stream_step(RawChunk<DT> (&cur)[kItems], RawChunk<DT> (&nxt)[kItems],
                                            TileOut<B> (&out)[kItems], bool have_prev, uint32_t s_prev,
                                            const void* __restrict__ x, uint32_t s0, uint32_t stride,
                                            Slices sl, float T, float rT, int tdyn, bool pz, const ScaleEntry* tab,
                                            u32x4* wave_lds, uint32_t* __restrict__ codes, uint8_t* __restrict__ scales,
                                            float* __restrict__ sse_out, float* __restrict__ clip_out)
{
    float v[kItems][8];
    __builtin_amdgcn_s_waitcnt(0x0F70);                              // vmcnt(0)
#pragma unroll
    for (int i = 0; i < kItems; ++i) widen<DT>(cur[i], v[i], wave_lds);
    __builtin_amdgcn_sched_barrier(0);
    if (have_prev) {                                                 // uniform
#pragma unroll
        for (int i = 0; i < kItems; ++i)
            store_slice<B>(out[i], s_prev + (uint32_t)i, sl, codes, scales, sse_out, CLIP ? clip_out : nullptr);
    }
    if (s0 + stride < sl.count) load_tile<DT>(nxt, x, s0 + stride, sl);            // uniform
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < kItems; ++i)
        process_chunk<B, FMT, FOUR6, TMODE, CLIP>(v[i], T, rT, tdyn, pz, tab, out[i].packed, out[i].code, out[i].sse,
                                                  out[i].clip);
}

// Main kernel: the complete chunks, grid-stride over workgroup tiles with two register buffers
// alternating between "being processed" and "in flight".
template <int DT, int B, int FMT, bool FOUR6, int TMODE, bool CLIP>
__global__ void __launch_bounds__(kThreads)
stream_kernel(const void* __restrict__ x, uint32_t n_slices, uint32_t last_chunks, float T_arg, int pz,
              const float* __restrict__ absmax_dev, float* __restrict__ t_out,
              uint32_t* __restrict__ codes, uint8_t* __restrict__ scales, float* __restrict__ sse_out,
              float* __restrict__ clip_out)
{
    __shared__ ScaleEntry tab[(FMT == kE8M0) ? 1 : 256];
    __shared__ u32x4 xpose[(DT == kF32) ? 2 * kThreads : 1];        // 2 KiB per wavefront, fp32 input only
    u32x4* wave_lds = xpose + ((DT == kF32) ? 2u * (threadIdx.x & ~63u) : 0u);

    const Slices sl{n_slices, last_chunks};
    const uint32_t stride = gridDim.x * (uint32_t)kItems;
    uint32_t s0 = blockIdx.x * (uint32_t)kItems;
    if (s0 >= sl.count) return;                                      // whole workgroup
    float T = T_arg;
    int tdyn = TMODE;
    if constexpr (TMODE == kDynT) {                  // T from the abs-max left in device memory, if there is one
        if (absmax_dev) T = tensor_scale_of<FMT>(*absmax_dev);
        tdyn = (T == 1.0f) ? kNoT : (fast_division_ok(T) ? kFastT : kSlowT);
        if (t_out && blockIdx.x == 0 && threadIdx.x == 0) *t_out = T;
    }
    const float rT = 1.0f / T;                                       // correctly rounded

    // the first tile's loads are in flight while the scale table is built
    RawChunk<DT> bufA[kItems], bufB[kItems];
#pragma unroll
    for (int i = 0; i < kItems; ++i) { bufA[i] = RawChunk<DT>{}; bufB[i] = RawChunk<DT>{}; }
    load_tile<DT>(bufA, x, s0, sl);
    if constexpr (FMT != kE8M0) fill_scale_table<FMT>(tab);
    TileOut<B> out[kItems];
    bool have_prev = false;
    uint32_t s_prev = s0;
    while (true) {
        stream_step<DT, B, FMT, FOUR6, TMODE, CLIP>(bufA, bufB, out, have_prev, s_prev, x, s0, stride, sl, T, rT, tdyn,
                                                    pz != 0, tab, wave_lds, codes, scales, sse_out, clip_out);
        have_prev = true;
        s_prev = s0;
        s0 += stride;
        if (s0 >= sl.count) break;
        stream_step<DT, B, FMT, FOUR6, TMODE, CLIP>(bufB, bufA, out, true, s_prev, x, s0, stride, sl, T, rT, tdyn,
                                                    pz != 0, tab, wave_lds, codes, scales, sse_out, clip_out);
        s_prev = s0;
        s0 += stride;
        if (s0 >= sl.count) break;
    }
#pragma unroll
    for (int i = 0; i < kItems; ++i)
        store_slice<B>(out[i], s_prev + (uint32_t)i, sl, codes, scales, sse_out, CLIP ? clip_out : nullptr);
}

// ---------------------------------------------------------------------------------------
// Several tensors in one launch.  A model's smaller matrices hold a few microseconds of work each,
// less than the start-up and drain of a launch; here up to kMaxBatch tensors share one grid.  The
// slices of all tensors form one index space (prefix sums in the kernel arguments); a workgroup
// resolves every tile to its tensor with a handful of scalar compares and then runs the very same
// pipeline step as the single-tensor kernel.  No per-tensor scale, no clipping output.
// ---------------------------------------------------------------------------------------
struct BatchArgs {
    const void* x[kMaxBatch];
    uint32_t* codes[kMaxBatch];
    uint8_t* scales[kMaxBatch];
    float* sse[kMaxBatch];
    uint32_t first[kMaxBatch + 1];        // first global slice of tensor t; first[count] = total
    uint32_t last[kMaxBatch];             // chunks in tensor t's last slice, 1 .. 256
    uint32_t count;
};

struct TileRef {                          // one tile = one slice of one tensor
    uint32_t t, s;                        // tensor, slice inside it
    Slices sl;
};

__device__ __forceinline__ TileRef locate(const BatchArgs& a, uint32_t g)
{
    uint32_t t = 0u;
#pragma unroll
    for (int k = 1; k < kMaxBatch; ++k) t += ((uint32_t)k < a.count && g >= a.first[k]) ? 1u : 0u;
    return TileRef{t, g - a.first[t], Slices{a.first[t + 1] - a.first[t], a.last[t]}};
}

template <int DT, int B, int FMT, bool FOUR6>
__device__ __forceinline__ void batch_step(RawChunk<DT> (&cur)[kItems], RawChunk<DT> (&nxt)[kItems],
                                           TileOut<B> (&out)[kItems], bool have_prev, TileRef prev,
                                           bool have_next, TileRef next, const BatchArgs& a, bool pz,
                                           const ScaleEntry* tab, u32x4* wave_lds)
{
    static_assert(kItems == 1, "one slice per tile");
    float v[8];
    __builtin_amdgcn_s_waitcnt(0x0F70);                              // vmcnt(0)
    widen<DT>(cur[0], v, wave_lds);
    __builtin_amdgcn_sched_barrier(0);
    if (have_prev)                                                   // uniform
        store_slice<B>(out[0], prev.s, prev.sl, a.codes[prev.t], a.scales[prev.t], a.sse[prev.t], nullptr);
    if (have_next) load_tile<DT>(nxt, a.x[next.t], next.s, next.sl); // uniform
    __builtin_amdgcn_sched_barrier(0);
    process_chunk<B, FMT, FOUR6, kNoT, false>(v, 1.0f, 1.0f, kNoT, pz, tab, out[0].packed, out[0].code, out[0].sse,
                                              out[0].clip);
}

// (Resolving the descriptors of a tile one pipeline step ahead, pointers included, was measured
// and is slower: it keeps three sets of pointers alive in scalar registers.)
template <int DT, int B, int FMT, bool FOUR6>
__global__ void __launch_bounds__(kThreads)
stream_batch_kernel(const BatchArgs a, int pz)
{
    __shared__ ScaleEntry tab[(FMT == kE8M0) ? 1 : 256];
    __shared__ u32x4 xpose[(DT == kF32) ? 2 * kThreads : 1];
    u32x4* wave_lds = xpose + ((DT == kF32) ? 2u * (threadIdx.x & ~63u) : 0u);

    const uint32_t total = a.first[a.count];
    const uint32_t stride = gridDim.x;
    uint32_t g = blockIdx.x;
    if (g >= total) return;                                          // whole workgroup

    RawChunk<DT> bufA[kItems], bufB[kItems];
    bufA[0] = RawChunk<DT>{};
    bufB[0] = RawChunk<DT>{};
    TileRef cur = locate(a, g), prev = cur, next = cur;
    load_tile<DT>(bufA, a.x[cur.t], cur.s, cur.sl);
    if constexpr (FMT != kE8M0) fill_scale_table<FMT>(tab);
    TileOut<B> out[kItems];
    bool have_prev = false;
    while (true) {
        bool have_next = g + stride < total;
        if (have_next) next = locate(a, g + stride);
        batch_step<DT, B, FMT, FOUR6>(bufA, bufB, out, have_prev, prev, have_next, next, a, pz != 0, tab, wave_lds);
        have_prev = true;
        prev = cur;
        if (!have_next) break;
        cur = next;
        g += stride;
        have_next = g + stride < total;
        if (have_next) next = locate(a, g + stride);
        batch_step<DT, B, FMT, FOUR6>(bufB, bufA, out, true, prev, have_next, next, a, pz != 0, tab, wave_lds);
        prev = cur;
        if (!have_next) break;
        cur = next;
        g += stride;
    }
    store_slice<B>(out[0], prev.s, prev.sl, a.codes[prev.t], a.scales[prev.t], a.sse[prev.t], nullptr);
}

// Ragged tail: when n is not a multiple of 8 (only possible for b = 2 or 4) the last
// `count` < 8 elements are handled by lane 0 of one wavefront, reading and writing element-wise.
template <int DT, int B, int FMT, bool FOUR6, int TMODE>
__global__ void __launch_bounds__(64)
stream_tail_kernel(const void* __restrict__ x, int64_t first, int count, float T_arg, int pz,
                   const float* __restrict__ absmax_dev, float* __restrict__ t_out,
                   uint8_t* __restrict__ codes, uint8_t* __restrict__ scales, float* __restrict__ sse_out,
                   float* __restrict__ clip_out)
{
    constexpr int NBLK = (B < 8) ? 8 / B : 1;
    __shared__ ScaleEntry tab[(FMT == kE8M0) ? 1 : 256];
    if constexpr (FMT != kE8M0) fill_scale_table<FMT>(tab);

    float v[8], sse_sel[4], clip_sel[4];
    uint32_t packed, code_out[NBLK];
    load_partial<DT>(x, first, (threadIdx.x == 0) ? count : 0, v);
    float T = T_arg;
    int tdyn = TMODE;
    if constexpr (TMODE == kDynT) {
        if (absmax_dev) T = tensor_scale_of<FMT>(*absmax_dev);
        tdyn = (T == 1.0f) ? kNoT : kSlowT;
        if (t_out && threadIdx.x == 0) *t_out = T;      // t_out is passed only when no main kernel runs
    }
    process_chunk<B, FMT, FOUR6, TMODE, true>(v, T, 1.0f / T, tdyn, pz != 0, tab, packed, code_out, sse_sel, clip_sel);
    if (threadIdx.x != 0) return;
    for (int i = 0; i < count / 2; ++i) codes[first / 2 + i] = (uint8_t)(packed >> (8 * i));
    if constexpr (B < 8) {
        for (int k = 0; k < NBLK; ++k) {
            if (k < count / B) {
                scales[first / B + k] = (uint8_t)code_out[k];
                if (sse_out) sse_out[first / B + k] = sse_sel[k];
                if (clip_out) clip_out[first / B + k] = clip_sel[k];
            }
        }
    }
}

// ------------------------------------------------------------------------------ dispatch

template <int DT, int B, int FMT, bool FOUR6>
static hipError_t launch_recipe(const StreamArgs& a, int pz)
{
    const int64_t n_full = a.n / 8;
    const int count = (int)(a.n - n_full * 8);
    // reciprocal-refined division only where its exactness argument holds; with the abs-max in
    // device memory the kernel makes the same choice itself
    // the variant that also writes the clipping-only SSE exists for the run-time mode only
    const int tmode = (a.absmax_dev || a.clip) ? kDynT : (a.T == 1.0f) ? kNoT : (fast_division_ok(a.T) ? kFastT : kSlowT);
    if (n_full > 0) {
        const int64_t slices = (n_full + kThreads - 1) / kThreads;
        const uint32_t n_slices = (uint32_t)slices;
        const uint32_t last = (uint32_t)(n_full - (slices - 1) * kThreads);
        const dim3 grid(stream_grid(((slices + kItems - 1) / kItems) * kThreads)), block(kThreads);
        uint32_t* codes = reinterpret_cast<uint32_t*>(a.codes);
#define MXQ_LAUNCH_STREAM(MODE, CLIP)                                                                 \
    hipLaunchKernelGGL((stream_kernel<DT, B, FMT, FOUR6, MODE, CLIP>), grid, block, 0, a.stream, a.x,       \
                       n_slices, last, a.T, pz, a.absmax_dev, a.t_out, codes, a.scales, a.sse, a.clip)
        if (a.clip) MXQ_LAUNCH_STREAM(kDynT, true);
        else if (tmode == kNoT) MXQ_LAUNCH_STREAM(kNoT, false);
        else if (tmode == kFastT) MXQ_LAUNCH_STREAM(kFastT, false);
        else if (tmode == kSlowT) MXQ_LAUNCH_STREAM(kSlowT, false);
        else MXQ_LAUNCH_STREAM(kDynT, false);
#undef MXQ_LAUNCH_STREAM
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if constexpr (B < 8) {
        if (count > 0) {
            float* t_out_tail = (n_full > 0) ? nullptr : a.t_out;
#define MXQ_LAUNCH_TAIL(MODE)                                                                         \
    hipLaunchKernelGGL((stream_tail_kernel<DT, B, FMT, FOUR6, MODE>), dim3(1), dim3(64), 0, a.stream, a.x,   \
                       n_full * 8, count, a.T, pz, a.absmax_dev, t_out_tail, a.codes, a.scales, a.sse, a.clip)
            if (tmode == kDynT) MXQ_LAUNCH_TAIL(kDynT);
            else if (tmode != kNoT) MXQ_LAUNCH_TAIL(kSlowT);
            else MXQ_LAUNCH_TAIL(kNoT);
#undef MXQ_LAUNCH_TAIL
        }
    }
    return hipGetLastError();
}

template <int DT, int B, int FMT>
static hipError_t launch_fmt(const StreamArgs& a)
{
    const bool four6 = (a.recipe == 2 || a.recipe == 3);
    const int pz = (a.recipe == 1 || a.recipe == 3) ? 1 : 0;
    if constexpr (FMT == kE8M0) {
        return launch_recipe<DT, B, FMT, false>(a, 0);
    } else {
        return four6 ? launch_recipe<DT, B, FMT, true>(a, pz) : launch_recipe<DT, B, FMT, false>(a, pz);
    }
}

template <int DT, int B>
static hipError_t launch_block(const StreamArgs& a)
{
    switch (a.scale_fmt) {
        case kE8M0: return launch_fmt<DT, B, kE8M0>(a);
        case kE4M3: return launch_fmt<DT, B, kE4M3>(a);
        default: return launch_fmt<DT, B, kUE5M3>(a);
    }
}

template <int DT>
static hipError_t launch_dt(const StreamArgs& a)
{
    switch (a.block) {
        case 2: return launch_block<DT, 2>(a);
        case 4: return launch_block<DT, 4>(a);
        case 8: return launch_block<DT, 8>(a);
        case 16: return launch_block<DT, 16>(a);
        case 32: return launch_block<DT, 32>(a);
        case 64: return launch_block<DT, 64>(a);
        default: return launch_block<DT, 128>(a);
    }
}

// ------------------------------------------------------------------------------ batch dispatch

template <int DT, int B, int FMT, bool FOUR6>
static hipError_t launch_batch_recipe(const StreamArgs* t, int count, int pz, hipStream_t stream)
{
    // complete chunks of up to kMaxBatch tensors per launch; ragged tails (b = 2, 4) one small launch each
    for (int i0 = 0; i0 < count; i0 += kMaxBatch) {
        BatchArgs a{};
        uint32_t n_t = 0u;
        uint64_t total = 0u;
        for (int i = i0; i < count && i < i0 + kMaxBatch; ++i) {
            const int64_t n_full = t[i].n / 8;
            if (n_full == 0) continue;
            const int64_t slices = (n_full + kThreads - 1) / kThreads;
            a.x[n_t] = t[i].x;
            a.codes[n_t] = reinterpret_cast<uint32_t*>(t[i].codes);
            a.scales[n_t] = t[i].scales;
            a.sse[n_t] = t[i].sse;
            a.first[n_t] = (uint32_t)total;
            a.last[n_t] = (uint32_t)(n_full - (slices - 1) * kThreads);
            total += (uint64_t)slices;
            ++n_t;
        }
        if (n_t > 0u) {
            a.first[n_t] = (uint32_t)total;                      // the host has bounded the sum below 2^32
            a.count = n_t;
            const dim3 grid(stream_grid((int64_t)total * kThreads)), block(kThreads);
            hipLaunchKernelGGL((stream_batch_kernel<DT, B, FMT, FOUR6>), grid, block, 0, stream, a, pz);
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    if constexpr (B < 8) {
        for (int i = 0; i < count; ++i) {
            const int64_t n_full = t[i].n / 8;
            const int cnt = (int)(t[i].n - n_full * 8);
            if (cnt > 0)
                hipLaunchKernelGGL((stream_tail_kernel<DT, B, FMT, FOUR6, kNoT>), dim3(1), dim3(64), 0, stream, t[i].x,
                                   n_full * 8, cnt, 1.0f, pz, (const float*)nullptr, (float*)nullptr, t[i].codes,
                                   t[i].scales, t[i].sse, (float*)nullptr);
        }
    }
    return hipGetLastError();
}

template <int DT, int B>
static hipError_t launch_batch_block(const StreamArgs* t, int count, hipStream_t stream)
{
    const int recipe = t[0].recipe;
    const bool four6 = (recipe == 2 || recipe == 3);
    const int pz = (recipe == 1 || recipe == 3) ? 1 : 0;
    switch (t[0].scale_fmt) {
        case kE8M0: return launch_batch_recipe<DT, B, kE8M0, false>(t, count, 0, stream);
        case kE4M3: return four6 ? launch_batch_recipe<DT, B, kE4M3, true>(t, count, pz, stream)
                                 : launch_batch_recipe<DT, B, kE4M3, false>(t, count, pz, stream);
        default: return four6 ? launch_batch_recipe<DT, B, kUE5M3, true>(t, count, pz, stream)
                              : launch_batch_recipe<DT, B, kUE5M3, false>(t, count, pz, stream);
    }
}

template <int DT>
static hipError_t launch_batch_dt(const StreamArgs* t, int count, hipStream_t stream)
{
    switch (t[0].block) {
        case 2: return launch_batch_block<DT, 2>(t, count, stream);
        case 4: return launch_batch_block<DT, 4>(t, count, stream);
        case 8: return launch_batch_block<DT, 8>(t, count, stream);
        case 16: return launch_batch_block<DT, 16>(t, count, stream);
        case 32: return launch_batch_block<DT, 32>(t, count, stream);
        case 64: return launch_batch_block<DT, 64>(t, count, stream);
        default: return launch_batch_block<DT, 128>(t, count, stream);
    }
}

// `t[0 .. count)`: validated tensors that share dtype, block, scale format and a streaming recipe.
hipError_t launch_stream_batch(const StreamArgs* t, int count, hipStream_t stream)
{
    if (count <= 0) return hipSuccess;
    return (t[0].dtype == kBF16) ? launch_batch_dt<kBF16>(t, count, stream) : launch_batch_dt<kF32>(t, count, stream);
}

hipError_t launch_stream(const StreamArgs& a)
{
    return (a.dtype == kBF16) ? launch_dt<kBF16>(a) : launch_dt<kF32>(a);
}

}  // namespace mxq
