// Device code of the capture-and-stage path for gfx950 (MI355X).
//
// capture_kernel is the producer of the paper's Ring^2 (section 4.2, steps 1-2;
// section 5 "Device-to-device kernel"; section 4.4 gather-compact): it copies the
// selected rows of one observed tensor into the device byte ring and publishes the
// record; or, in one launch, the rows of up to kMaxBatch tensors of one layout that share a
// selection, one record each, laid down as single launches in the same order would (a
// launch costs microseconds whatever it moves, and only more bytes per launch amortise
// that).  The paper's kernel (1-64 blocks, grid-stride 16-byte copies, last block
// publishes) is prior art for other hardware; here
//   * every workgroup rebuilds the per-request prefix sums in LDS with wavefront
//     shuffle scans, so row -> (request, token) needs no pre-pass launch;
//   * rows are read with 16-byte vector loads and written with non-temporal
//     16-byte stores (the ring is not read again by the GPU, so it should not
//     displace the model's working set from the 4 MB per-XCD L2);
//   * downcasts and fp32 row summaries happen in the same pass, summaries by
//     wavefront shuffles (no matrix cores: nothing here is a contraction);
//   * the record's place in the ring comes from a device-resident head, and the
//     drop-newest decision from the drained mark as an earlier launch read it from a
//     word the host keeps current, both double buffered along the chain of launches:
//     every workgroup reads the same values with no atomic and no workgroup has to be
//     "the last one" (a compare-and-swap on one word from a thousand workgroups
//     measured 7 us here);
//   * there is no fence and no completion counter in the kernel: on this GPU a
//     device-scope fence writes back a whole L2, once per wavefront that issues it
//     (measured: 19 us for a 64-workgroup capture, 300 us for 2048 workgroups).
//     Workgroup 0 writes where the head stands into this launch's commit slot in
//     device memory, and the host fetches a slot only behind an event recorded after
//     the launch (the kernel-end release makes payload and slot visible);
//   * a small capture is a chain of dependent trips to memory and little else, so every
//     kernel here fetches its argument lines, its control words and its first rows in
//     as few trips as their dependencies allow (see touch_argument_lines, fetch_control,
//     lds_barrier), and the common small shapes have a short straight-line kernel of
//     their own (capture_decode_kernel).
#include "dmi_internal.h"
#include "dmi_debug.h"

#include <hip/hip_ext.h>
#include <hip/hip_fp16.h>

#include <cstring>

namespace dmi {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

enum OutMode { OUT_RAW = 0, OUT_FP16 = 1, OUT_FP8 = 2, OUT_NONE = 3 };

// ---------------------------------------------------------------- atomics
__device__ __forceinline__ uint64_t ld_agent(const uint64_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// a word the host writes (pinned host memory): every read crosses the host link
__device__ __forceinline__ uint64_t ld_system(const uint64_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}
__device__ __forceinline__ void st_agent(uint64_t *p, uint64_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---------------------------------------------------------------- wavefront helpers
// Workgroup barrier that orders LDS traffic only.  __syncthreads() also makes every
// wavefront wait until all of its global stores have been acknowledged, a round trip to
// memory of a microsecond or more; values handed over through LDS do not need that, and
// nothing here reads global memory written by another lane of the same launch.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v, uint32_t lane)
{
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t t = __shfl_up(v, d, 64);
        if (lane >= (uint32_t)d) v += t;
    }
    return v;
}
// Wavefront reductions with DPP (data-parallel primitives: the cross-lane operand rides on the
// ALU instruction, no trip through LDS).  quad_perm / row_half_mirror / row_mirror combine the 16
// lanes of a row, row_bcast15 / row_bcast31 carry row totals forward; lane 63 ends up with the
// total, which is read back as a scalar.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, false);
}
__device__ __forceinline__ float wave_sum(float v)
{
    v += __uint_as_float(dpp_u32<0xB1, 0xF>(__float_as_uint(v)));      // quad_perm [1,0,3,2]
    v += __uint_as_float(dpp_u32<0x4E, 0xF>(__float_as_uint(v)));      // quad_perm [2,3,0,1]
    v += __uint_as_float(dpp_u32<0x141, 0xF>(__float_as_uint(v)));     // row_half_mirror
    v += __uint_as_float(dpp_u32<0x140, 0xF>(__float_as_uint(v)));     // row_mirror
    v += __uint_as_float(dpp_u32<0x142, 0xA>(__float_as_uint(v)));     // row_bcast15 into rows 1, 3
    v += __uint_as_float(dpp_u32<0x143, 0xC>(__float_as_uint(v)));     // row_bcast31 into rows 2, 3
    return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(v), 63));
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    uint32_t o;
    o = dpp_u32<0xB1, 0xF>(v);  v = o > v ? o : v;
    o = dpp_u32<0x4E, 0xF>(v);  v = o > v ? o : v;
    o = dpp_u32<0x141, 0xF>(v); v = o > v ? o : v;
    o = dpp_u32<0x140, 0xF>(v); v = o > v ? o : v;
    o = dpp_u32<0x142, 0xA>(v); v = o > v ? o : v;
    o = dpp_u32<0x143, 0xC>(v); v = o > v ? o : v;
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// ---------------------------------------------------------------- conversions
// bf16 -> fp8 E4M3FN (OCP: bias 7, max 448, no inf, S.1111.111 NaN), round to
// nearest even, saturating.  Integer arithmetic on the bf16 bit pattern; used on the
// element-wise path (rows that cannot be moved as 16-byte vectors).
__device__ __forceinline__ uint32_t bf16_to_fp8(uint32_t b)
{
    const uint32_t sign = (b >> 8) & 0x80u;
    const uint32_t a = b & 0x7FFFu;
    const uint32_t e = a >> 7;
    uint32_t code;
    if (e >= 121u) {
        // normal in fp8 (|x| >= 2^-6): rebias 127 -> 7, drop 4 mantissa bits with RNE
        const uint32_t x = a - (120u << 7);
        code = (x + 7u + ((x >> 4) & 1u)) >> 4;
        code = code > 0x7Eu ? 0x7Eu : code;
    } else {
        // fp8 subnormal: |x| / 2^-9 = (128 + m) >> (125 - e), RNE; vanishes for shifts > 8
        const uint32_t sh = 125u - e;
        const uint32_t s = sh > 9u ? 9u : sh;
        const uint32_t v = 128u + (a & 0x7Fu);
        code = (v + (1u << (s - 1u)) - 1u + ((v >> s) & 1u)) >> s;
    }
    if (a > 0x7F80u) code = 0x7Fu;
    return sign | code;
}

// Two bf16 (one 32-bit word) -> two fp8 E4M3FN codes in the low or high half of `acc`.
// gfx950's packed convert rounds to nearest even into the OCP format, subnormals
// included, but does not saturate (values that round beyond 448, and infinities, come
// out as NaN) and drops a NaN's sign; so magnitudes are clamped to 448 first with a
// packed 16-bit minimum, and words holding a NaN are patched afterwards.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef short s16x2_t __attribute__((ext_vector_type(2)));
typedef unsigned short u16x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ s16x2_t bf16x2_to_fp8x2(uint32_t w, s16x2_t acc, bool hi)
{
    const uint32_t mag = w & 0x7FFF7FFFu;
    const u16x2_t lim = {0x43E0u, 0x43E0u};                                   // 448.0
    const u16x2_t cl = __builtin_elementwise_min(__builtin_bit_cast(u16x2_t, mag), lim);
    const uint32_t x = __builtin_bit_cast(uint32_t, cl) | (w & 0x80008000u);
    const bf16x2_t v = __builtin_bit_cast(bf16x2_t, x);
    acc = hi ? __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(acc, v, 1.0f, true)
             : __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(acc, v, 1.0f, false);
    const u16x2_t inf = {0x7F80u, 0x7F80u};
    const u16x2_t over = __builtin_elementwise_sub_sat(__builtin_bit_cast(u16x2_t, mag), inf);
    if (__builtin_bit_cast(uint32_t, over) != 0u) {                           // a NaN: sign | 0x7F
        uint32_t pair = (uint32_t)(unsigned short)(hi ? acc.y : acc.x);
        if (over.x) pair = (pair & 0xFF00u) | ((w >> 8) & 0x80u) | 0x7Fu;
        if (over.y) pair = (pair & 0x00FFu) | (((w >> 24) & 0x80u) << 8) | 0x7F00u;
        if (hi) acc.y = (short)pair; else acc.x = (short)pair;
    }
    return acc;
}

// bf16 -> fp16: exact widening to f32, then the hardware's round-to-nearest-even
// convert (overflow to inf, gradual underflow); NaN -> sign | 0x7E00.
__device__ __forceinline__ uint32_t bf16_to_fp16(uint32_t b)
{
    const float f = __uint_as_float(b << 16);
    uint32_t h = (uint32_t)__half_as_ushort(__float2half_rn(f));
    if ((b & 0x7FFFu) > 0x7F80u) h = ((b >> 15) << 15) | 0x7E00u;
    return h;
}

__device__ __forceinline__ float widen16(uint32_t bits, uint32_t src_dtype)
{
    return src_dtype == 1u ? __uint_as_float(bits << 16)
                           : __half2float(__ushort_as_half((unsigned short)bits));
}

// ---------------------------------------------------------------- units
// A unit is what one lane moves per access: 16 source bytes on the vector path,
// one element on the element path.
template <int NB> struct UnitT;
template <> struct UnitT<16> { typedef u32x4 T; };
template <> struct UnitT<8>  { typedef u32x2 T; };
template <> struct UnitT<4>  { typedef uint32_t T; };
template <> struct UnitT<2>  { typedef uint16_t T; };
template <> struct UnitT<1>  { typedef uint8_t T; };

struct RingW {
    uint8_t *ring;
    uint64_t cap;
    uint64_t base;      // physical offset of the record's first byte
};

template <typename T>
__device__ __forceinline__ void ring_store(const RingW &w, uint64_t off, T v)
{
    uint64_t p = w.base + off;
    if (p >= w.cap) p -= w.cap;
    // streaming stores for the vectors a wavefront lays down as whole lines; small scalars (a
    // summary value per workgroup, pad bytes) are left to L2 to merge: as streaming stores of a
    // fraction of a line they cost a launch microseconds
    if constexpr (sizeof(T) >= 8) __builtin_nontemporal_store(v, reinterpret_cast<T *>(w.ring + p));
    else *reinterpret_cast<T *>(w.ring + p) = v;
}

// Per-lane partial row summaries.  Sum of squares and sum are fp32; the largest magnitude is
// kept as the bit pattern of |x| in the source format (sign-magnitude formats order like
// unsigned integers, and a NaN, whose pattern is above infinity's, wins the maximum and so
// surfaces as NaN).  16-bit sources keep two independent 16-bit maxima in one word.
struct Accum {
    float ss, s;
    uint32_t am;
};

typedef _Float16 h16x2_t __attribute__((ext_vector_type(2)));

// two 16-bit elements in one word: v_dot2 does x0*x0 + x1*x1 + acc (and x0 + x1 + acc with a
// vector of ones) without unpacking; v_pk_max_u16 tracks the magnitudes
__device__ __forceinline__ void accum_pair(Accum &a, uint32_t w, bool is_bf16)
{
    if (is_bf16) {
        const bf16x2_t x = __builtin_bit_cast(bf16x2_t, w);
        const bf16x2_t one = __builtin_bit_cast(bf16x2_t, 0x3F803F80u);
        a.ss = __builtin_amdgcn_fdot2_f32_bf16(x, x, a.ss, false);
        a.s = __builtin_amdgcn_fdot2_f32_bf16(x, one, a.s, false);
    } else {
        const h16x2_t x = __builtin_bit_cast(h16x2_t, w);
        const h16x2_t one = __builtin_bit_cast(h16x2_t, 0x3C003C00u);
        a.ss = __builtin_amdgcn_fdot2(x, x, a.ss, false);
        a.s = __builtin_amdgcn_fdot2(x, one, a.s, false);
    }
    a.am = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2_t, a.am),
                                                                  __builtin_bit_cast(u16x2_t, w & 0x7FFF7FFFu)));
}

__device__ __forceinline__ void accum_f32(Accum &a, uint32_t bits)
{
    const float x = __uint_as_float(bits);
    a.ss = fmaf(x, x, a.ss);
    a.s += x;
    const uint32_t m = bits & 0x7FFFFFFFu;
    a.am = m > a.am ? m : a.am;
}

// one 16-bit element (element-wise path)
__device__ __forceinline__ void accum_16(Accum &a, uint32_t bits, uint32_t src_dtype)
{
    const float x = widen16(bits, src_dtype);
    a.ss = fmaf(x, x, a.ss);
    a.s += x;
    const uint32_t m = bits & 0x7FFFu;
    a.am = m > a.am ? m : a.am;
}

// the lane's magnitude maximum as one value comparable across lanes
template <int ES_IN, int VEC>
__device__ __forceinline__ uint32_t fold_am(uint32_t am)
{
    if constexpr (ES_IN == 2 && VEC == 8) return (am & 0xFFFFu) > (am >> 16) ? (am & 0xFFFFu) : (am >> 16);
    else return am;
}

__device__ __forceinline__ float am_value(uint32_t m, uint32_t src_dtype)
{
    if (src_dtype == 3u) return __uint_as_float(m);
    return widen16(m, src_dtype);
}

// Convert one source unit and store it; optionally accumulate the row summaries.
template <int ES_IN, int VEC, int OUT, bool SUMM>
__device__ __forceinline__ void emit_unit(const RingW &w, uint64_t out_off,
                                          typename UnitT<ES_IN * VEC>::T v, uint32_t src_dtype,
                                          Accum &acc)
{
    if constexpr (ES_IN == 2 && VEC == 8) {
        uint32_t wd[4] = {v.x, v.y, v.z, v.w};
        if constexpr (SUMM) {
            const bool is_bf16 = src_dtype == 1u;
#pragma unroll
            for (int k = 0; k < 4; k++) accum_pair(acc, wd[k], is_bf16);
        }
        if constexpr (OUT == OUT_RAW) {
            ring_store<u32x4>(w, out_off, v);
        } else if constexpr (OUT == OUT_FP16) {
            u32x4 o;
            uint32_t ow[4];
#pragma unroll
            for (int k = 0; k < 4; k++)
                ow[k] = bf16_to_fp16(wd[k] & 0xFFFFu) | (bf16_to_fp16(wd[k] >> 16) << 16);
            o.x = ow[0]; o.y = ow[1]; o.z = ow[2]; o.w = ow[3];
            ring_store<u32x4>(w, out_off, o);
        } else if constexpr (OUT == OUT_FP8) {
            s16x2_t lo = {0, 0}, hi = {0, 0};
            lo = bf16x2_to_fp8x2(wd[0], lo, false);
            lo = bf16x2_to_fp8x2(wd[1], lo, true);
            hi = bf16x2_to_fp8x2(wd[2], hi, false);
            hi = bf16x2_to_fp8x2(wd[3], hi, true);
            u32x2 o;
            o.x = __builtin_bit_cast(uint32_t, lo);
            o.y = __builtin_bit_cast(uint32_t, hi);
            ring_store<u32x2>(w, out_off, o);
        }
    } else if constexpr (ES_IN == 4 && VEC == 4) {
        if constexpr (SUMM) {
            accum_f32(acc, v.x);
            accum_f32(acc, v.y);
            accum_f32(acc, v.z);
            accum_f32(acc, v.w);
        }
        if constexpr (OUT == OUT_RAW) ring_store<u32x4>(w, out_off, v);
    } else if constexpr (ES_IN == 2) {      // one 2-byte element
        const uint32_t b = v;
        if constexpr (SUMM) accum_16(acc, b, src_dtype);
        if constexpr (OUT == OUT_RAW) ring_store<uint16_t>(w, out_off, (uint16_t)b);
        else if constexpr (OUT == OUT_FP16) ring_store<uint16_t>(w, out_off, (uint16_t)bf16_to_fp16(b));
        else if constexpr (OUT == OUT_FP8) ring_store<uint8_t>(w, out_off, (uint8_t)bf16_to_fp8(b));
    } else {                                // one 4-byte element
        if constexpr (SUMM) accum_f32(acc, v);
        if constexpr (OUT == OUT_RAW) ring_store<uint32_t>(w, out_off, v);
    }
}

template <int ES_IN, int VEC, int OUT>
__host__ __device__ constexpr uint32_t out_unit_bytes()
{
    return OUT == OUT_NONE ? 0u : OUT == OUT_FP8 ? (uint32_t)VEC : (uint32_t)(ES_IN * VEC);
}

// ---------------------------------------------------------------- LDS layout
struct LdsMap {
    uint32_t hdr, heads, red, bcast, pref, btot, pref_all, btot_all, tab, rb, total_words;
};

__host__ __device__ inline LdsMap lds_map(uint32_t n_reqs, bool index_mode, bool table_in_lds)
{
    LdsMap m;
    const uint32_t nb = (n_reqs + 63u) / 64u;
    uint32_t p = 0;
    m.hdr = p; p += 16;
    m.heads = p; p += 8;
    m.red = p; p += 12;
    m.bcast = p; p += 12;          // head, tail, ring offset of the head, policy flags, seq, step id
    m.pref = p; p += n_reqs + 1;
    m.btot = p; p += nb + 1;
    m.pref_all = p; m.btot_all = p;
    if (index_mode) { p += n_reqs + 1; m.btot_all = p; p += nb + 1; }
    p = (p + 3u) & ~3u;
    m.tab = p; m.rb = p;
    if (table_in_lds) { p += 4 * n_reqs; m.rb = p; p += n_reqs; }
    m.total_words = p;
    return m;
}

uint32_t capture_lds_bytes(uint32_t n_reqs, bool index_mode, bool table_in_lds)
{
    return lds_map(n_reqs, index_mode, table_in_lds).total_words * 4u;
}

// Where one output row comes from.
struct RowRef {
    const uint8_t *base;    // dense: first byte of the row; paged: first byte of the slot
    uint64_t ok;            // 0 if a device-side index left the source (a full word: the struct
                            // is copied around and should stay in registers)
};

// Control words of one launch, fetched by one lane per workgroup.  Every load is issued
// before any result is used, whether or not this launch needs it: loads issued together
// cost one trip to memory, loads issued as their conditions become known cost one each.
struct RawControl {
    uint64_t head, tail_for, sp_seq, sp_step, sp_floor;
    uint64_t cap[3], drop[3];
    uint32_t sp_flags;
};
struct Control {
    uint64_t head, tail, seq, step_id;
    uint32_t flags;
};

// Issues the loads and touches none of the results, so that the caller can put more
// loads behind them before the first wait.
__device__ __forceinline__ RawControl fetch_control(const DevCtrl *c, uint32_t par, const StepParams *step)
{
    RawControl r;
    // a launch outside a replayable step reads (and ignores) the head of the control block instead
    const StepParams *spp = step ? step : reinterpret_cast<const StepParams *>(c);
    r.head = c->head[par];
    r.tail_for = c->tail_for[par];
    r.sp_seq = spp->seq_base; r.sp_step = spp->step_id; r.sp_floor = spp->tail_floor;
    r.sp_flags = spp->flags;
    r.cap[0] = c->captured_records; r.cap[1] = c->captured_rows; r.cap[2] = c->captured_bytes;
    r.drop[0] = c->dropped_records; r.drop[1] = c->dropped_rows; r.drop[2] = c->dropped_bytes;
    return r;
}

__device__ __forceinline__ Control resolve_control(const RawControl &r, bool in_step, uint32_t node,
                                                   uint64_t tail_floor, uint64_t seq, uint64_t step_id, uint32_t flags)
{
    Control o;
    o.head = r.head;
    o.seq = in_step ? r.sp_seq + node : seq;
    o.step_id = in_step ? r.sp_step : step_id;
    o.flags = in_step ? r.sp_flags : flags;
    const uint64_t floor = in_step ? r.sp_floor : tail_floor;
    o.tail = (o.flags & kStepDropNewest) && r.tail_for > floor ? r.tail_for : floor;
    return o;
}

// Fetch every line of a by-value kernel argument block now, together, along with this
// workgroup's entry of the batch block (its tensor and observation point).
template <typename T>
__device__ __forceinline__ void touch_argument_lines(const T &a, const uint8_t *src, uint32_t point)
{
    const uint32_t *p = reinterpret_cast<const uint32_t *>(&a);
    constexpr uint32_t n = (sizeof(T) + 63u) / 64u;
    static_assert(n <= 10, "argument block larger than expected");
    auto at = [p](uint32_t line) { return p[(line < n ? line : n - 1u) * 16u]; };
    asm volatile("" ::"s"(at(0)), "s"(at(1)), "s"(at(2)), "s"(at(3)), "s"(at(4)), "s"(at(5)), "s"(at(6)), "s"(at(7)),
                 "s"(at(8)), "s"(at(9)), "s"((uint32_t)(uintptr_t)src), "s"((uint32_t)((uintptr_t)src >> 32)), "s"(point));
}

// ---------------------------------------------------------------- capture kernel
template <int ES_IN, int VEC, int OUT, bool SUMM>
__global__ void __launch_bounds__(kThreads) capture_kernel(const CaptureKernelArgs a, const BatchArgs b)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
    const uint32_t y = blockIdx.y;                  // which tensor of the batch this workgroup works on
    const uint8_t *const src = b.src[y];
    const uint32_t point_id = b.point[y];
    touch_argument_lines(a, src, point_id);         // all of it in one trip, not one by one
    constexpr uint32_t NB_IN = ES_IN * VEC;
    constexpr uint32_t NB_OUT = out_unit_bytes<ES_IN, VEC, OUT>();
    typedef typename UnitT<NB_IN>::T unit_t;

    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t n_reqs = a.n_reqs;
    const bool index_mode = a.row_index != nullptr;
    const bool simple = a.simple != 0;          // no keep mask and one row per request
    const LdsMap m = lds_map(simple ? 0u : n_reqs, index_mode, a.table_in_lds != 0);
    uint32_t *pref = lds + m.pref, *btot = lds + m.btot;
    uint32_t *pref_all = lds + m.pref_all, *btot_all = lds + m.btot_all;
    uint4 *ltab = reinterpret_cast<uint4 *>(lds + m.tab);
    uint32_t *lrb = lds + m.rb;
    const uint32_t nb = (n_reqs + 63u) / 64u;
    const uint32_t par = a.par_in;

    // -- control words: lane 0 of the last wavefront fetches head, tail copy, running counters
    //    and (for a replayable step) the step's parameters, all at once and whether or not this
    //    workgroup will need them, while the first wavefronts start on the request table.
    //    Every dependent trip to memory costs most of a microsecond, and a small capture is
    //    made of little else.  Head and tail are double buffered along the chain of launches:
    //    this launch reads what the previous one left and writes the other copy, so the
    //    values are the same for every workgroup with no atomic and no waiting.
    constexpr uint32_t kCtlTid = kThreads - 64u;
    uint64_t cnt_cap[3] = {0, 0, 0}, cnt_drop[3] = {0, 0, 0}, tail_now = 0, seq = a.seq;
    RawControl raw = {};
    if (tid == kCtlTid)     // issued here, used just before the barrier below
        raw = fetch_control(a.ctrl, par, a.step);
    auto publish_control = [&]() {
        const Control ct = resolve_control(raw, a.step != nullptr, a.node, a.tail_floor, a.seq, a.step_id,
                                           a.drop_newest);
        seq = ct.seq;
        for (int i = 0; i < 3; i++) { cnt_cap[i] = raw.cap[i]; cnt_drop[i] = raw.drop[i]; }
        const uint64_t base = ct.head % a.cap;
        lds[m.bcast + 4] = (uint32_t)base;
        lds[m.bcast + 5] = (uint32_t)(base >> 32);
        lds[m.bcast + 0] = (uint32_t)ct.head;
        lds[m.bcast + 1] = (uint32_t)(ct.head >> 32);
        lds[m.bcast + 2] = (uint32_t)ct.tail;
        lds[m.bcast + 3] = (uint32_t)(ct.tail >> 32);
        lds[m.bcast + 6] = ct.flags;
        lds[m.bcast + 8] = (uint32_t)ct.seq;
        lds[m.bcast + 9] = (uint32_t)(ct.seq >> 32);
        lds[m.bcast + 10] = (uint32_t)ct.step_id;
        lds[m.bcast + 11] = (uint32_t)(ct.step_id >> 32);
    };
    if (tid < 8) lds[m.heads + tid] = a.heads_sel[tid];

    if (!simple) {
        // -- per-request kept row counts -> exclusive prefix sums (wavefront shuffle scans)
        for (uint32_t b = wave; b < nb; b += kThreads / 64u) {
            const uint32_t r = b * 64u + lane;
            uint32_t cnt = 0, cnt_all = 0;
            if (r < n_reqs) {
                uint4 e = a.req_table[r];
                cnt_all = e.w;
                const bool keep = a.keep_mask ? a.keep_mask[r] != 0 : true;
                cnt = keep ? cnt_all : 0u;
                if (a.table_in_lds) {
                    e.w = cnt;
                    ltab[r] = e;
                    lrb[r] = a.row0[r];
                }
            }
            const uint32_t inc = wave_incl_scan(cnt, lane);
            if (r < n_reqs) pref[r] = inc - cnt;
            if (lane == 63u) { btot[b] = inc; if (nb == 1u) pref[n_reqs] = inc; }
            if (index_mode) {
                const uint32_t inc_all = wave_incl_scan(cnt_all, lane);
                if (r < n_reqs) pref_all[r] = inc_all - cnt_all;
                if (lane == 63u) { btot_all[b] = inc_all; if (nb == 1u) pref_all[n_reqs] = inc_all; }
            }
        }
        // up to 64 requests: one wavefront has done it all, and the barrier in front of the
        // geometry below is the only one needed
        if (nb != 1u) {
        lds_barrier();
        if (wave == 0) {
            uint32_t carry = 0, carry_all = 0;
            for (uint32_t b0 = 0; b0 < nb; b0 += 64u) {
                const uint32_t b = b0 + lane;
                const uint32_t v = b < nb ? btot[b] : 0u;
                const uint32_t inc = wave_incl_scan(v, lane);
                if (b < nb) btot[b] = carry + inc - v;
                carry += __shfl(inc, 63, 64);
                if (index_mode) {
                    const uint32_t va = b < nb ? btot_all[b] : 0u;
                    const uint32_t ia = wave_incl_scan(va, lane);
                    if (b < nb) btot_all[b] = carry_all + ia - va;
                    carry_all += __shfl(ia, 63, 64);
                }
            }
            if (lane == 0) {
                btot[nb] = carry;
                if (index_mode) btot_all[nb] = carry_all;
            }
        }
        lds_barrier();
        for (uint32_t r = tid; r < n_reqs; r += kThreads) {
            pref[r] += btot[r >> 6];
            if (index_mode) pref_all[r] += btot_all[r >> 6];
        }
        if (tid == 0) {
            pref[n_reqs] = btot[nb];
            if (index_mode) pref_all[n_reqs] = btot_all[nb];
        }
        }
    }
    // -- decode-shaped selections (no mask, one row per request, dense): the first work
    //    item's rows do not depend on anything computed above, so their loads are issued
    //    now and travel together with the control fetch instead of behind it
    constexpr uint32_t U = 4;                               // loads in flight per lane
    constexpr uint32_t CH = U * kThreads;                   // units per long-row work item
    const uint32_t rpw = SUMM ? a.rows_per_wg : 1u;
    const uint32_t gsz = kThreads / rpw;                    // lanes per row (summary passes)
    const uint32_t sub = tid / gsz, l = tid - sub * gsz;
    const uint32_t cpr = (a.units_per_row + CH - 1u) / CH;  // long-row items per row
    unit_t pre_v[U];
    RowRef pre_ref = {nullptr, 0};
    bool pre = false;
    const bool multi_row_items = a.units_per_row < CH && CH % a.units_per_row == 0u;
    // (not in a launch of several records some of which may turn out to be dropped: a dropped
    // record's rows would have been read for nothing)
    const bool may_drop_some = a.n_batch > 1u && (a.drop_newest != 0u || a.step != nullptr);
    if (simple && !a.paged && !may_drop_some &&
        (SUMM || (OUT != OUT_NONE && a.units_per_row >= kThreads && !multi_row_items))) {
        uint32_t g, c_begin, stride;
        if constexpr (SUMM) { g = blockIdx.x * rpw + sub; c_begin = l; stride = gsz; }
        else { g = blockIdx.x / cpr; c_begin = (blockIdx.x - g * cpr) * CH + tid; stride = kThreads; }
        if (g < n_reqs) {
            const int64_t row = index_mode ? (int64_t)a.row_index[g] : (int64_t)a.row0[g];
            pre_ref.ok = row >= 0 && row < a.n_src_rows;
            pre_ref.base = src + (pre_ref.ok ? row : 0) * a.row_stride_b;
#pragma unroll
            for (uint32_t k = 0; k < U; k++) {
                const uint32_t c = c_begin + k * stride;
                const bool want = pre_ref.ok && c < a.units_per_row;
                const uint8_t *p = want ? pre_ref.base + (uint64_t)c * NB_IN : reinterpret_cast<const uint8_t *>(a.ctrl);
                pre_v[k] = *reinterpret_cast<const unit_t *>(p);     // zeroed where it is used if not wanted
            }
            pre = true;
        }
    }
    if (tid == kCtlTid) {
        // the drained-up-to mark for the next launch's drop decision: workgroup 0 reads it where
        // the host keeps it (a read across the host link, issued after every other load of this
        // lane so that none of them queues behind it; nothing in this launch waits for it but
        // the closing stores of this one lane)
        const uint64_t *ts = blockIdx.x == 0 && y == 0 && a.tail_src ? a.tail_src : &a.ctrl->tail;
        tail_now = ld_system(ts);
        publish_control();
    }
    lds_barrier();

    // -- record geometry
    const uint32_t n_rows = simple ? n_reqs : pref[n_reqs];
    const uint32_t es_out = OUT == OUT_NONE ? 0u : OUT == OUT_FP8 ? 1u : (uint32_t)ES_IN;
    const uint64_t table_bytes = ((uint64_t)n_reqs * 16u + 63u) & ~63ull;
    const uint64_t payload_bytes = (uint64_t)n_rows * a.row_elems * es_out;
    const uint64_t off_payload = 64u + table_bytes;
    const uint64_t off_sum = off_payload + ((payload_bytes + 63u) & ~63ull);
    const uint64_t sum_arr = ((uint64_t)n_rows * 4u + 63u) & ~63ull;
    const uint32_t n_sum = __popc(a.summary_mask & 7u);
    const uint64_t record_bytes = off_sum + (uint64_t)n_sum * sum_arr;

    // Record y of the launch lies y records behind the head the launch found: all records of a
    // batch have the same size, so record y fits iff the y before it did, and then they were kept.
    const uint64_t head0 = (uint64_t)lds[m.bcast + 0] | ((uint64_t)lds[m.bcast + 1] << 32);
    const uint64_t head = head0 + (uint64_t)y * record_bytes;
    const uint32_t flags = lds[m.bcast + 6];
    const bool publisher = blockIdx.x == 0 && y == 0 && tid == kCtlTid;
    if (flags & kStepSkip) {
        // a sampled-out replay: no record, no sequence number; the chain of head and tail
        // copies still has to reach the next launch
        if (publisher) {
            a.ctrl->head[par ^ 1u] = head0;
            a.ctrl->tail_for[par ^ 1u] = tail_now > raw.tail_for ? tail_now : raw.tail_for;
        }
        return;
    }
    const uint64_t tail = (uint64_t)lds[m.bcast + 2] | ((uint64_t)lds[m.bcast + 3] << 32);
    const bool drop_newest = (flags & kStepDropNewest) != 0;
    const bool dropped = a.force_drop != 0u || (drop_newest && head - tail + record_bytes > a.cap);

    // ---- publish: one lane of the launch leaves head, tail and counters for the next launch and
    //      fills the commit slot of the launch's last record, early, so that it overlaps the copy.
    //      Everything here is device memory; it becomes visible to the next launch and to the copy
    //      that fetches the slot with the kernel-end release.
    if (publisher) {
        DevCtrl *c = a.ctrl;
        const uint64_t nb_rec = gridDim.y;
        uint64_t n_fit = nb_rec;
        if (drop_newest) {
            const uint64_t used = head0 - tail;
            n_fit = used < a.cap ? (a.cap - used) / record_bytes : 0u;
            n_fit = n_fit < nb_rec ? n_fit : nb_rec;
        }
        if (a.force_drop) n_fit = 0;
        const uint64_t n_drop = nb_rec - n_fit + a.n_tail_drop;
        const uint64_t new_head = head0 + n_fit * record_bytes;
        if (n_drop) {
            cnt_drop[0] += n_drop; cnt_drop[1] += n_drop * n_rows; cnt_drop[2] += n_drop * record_bytes;
            c->dropped_records = cnt_drop[0]; c->dropped_rows = cnt_drop[1]; c->dropped_bytes = cnt_drop[2];
        }
        if (n_fit) {
            cnt_cap[0] += n_fit; cnt_cap[1] += n_fit * n_rows; cnt_cap[2] += n_fit * record_bytes;
            c->captured_records = cnt_cap[0]; c->captured_rows = cnt_cap[1]; c->captured_bytes = cnt_cap[2];
        }
        c->head[par ^ 1u] = new_head;
        c->tail_for[par ^ 1u] = tail_now > raw.tail_for ? tail_now : raw.tail_for;
        const uint64_t last_seq = seq + nb_rec + a.n_tail_drop - 1u;
        // (a loop of one lane over a uniform index: the points come straight out of the argument block)
        for (uint32_t i = 0; i < a.n_tail_drop; i++)
            atomicAdd(&c->point_drops[b.point[nb_rec + i] & 4095u], 1u);
        CommitSlot *h = a.step ? &c->slots[last_seq % kCommitSlots] : a.cslot;
        h->head = new_head;
        h->captured_records = cnt_cap[0];
        h->captured_rows = cnt_cap[1];
        h->captured_bytes = cnt_cap[2];
        h->dropped_records = cnt_drop[0];
        h->dropped_rows = cnt_drop[1];
        h->dropped_bytes = cnt_drop[2];
        h->seq_plus1 = last_seq + 1u;
    }
    if (dropped && blockIdx.x == 0 && tid == kCtlTid)
        atomicAdd(&a.ctrl->point_drops[point_id & 4095u], 1u);

    // Whoever issued a launch of several records made sure they fit the ring together (or the
    // ones that do not are dropped), so y records past the head are less than one lap away.
    RingW w;
    w.ring = a.ring;
    w.cap = a.cap;
    w.base = ((uint64_t)lds[m.bcast + 4] | ((uint64_t)lds[m.bcast + 5] << 32)) + (uint64_t)y * record_bytes;
    if (w.base >= w.cap) w.base -= w.cap;

    // row g -> request r (largest r with pref[r] <= g; requests with no rows are skipped
    // because their successor shares the same prefix) -> source location
    // (LDS is read through a pointer that says so: where the table may live either in LDS or
    // in global memory the compiler otherwise merges the two reads into one untyped load,
    // which counts as a global one and makes every wait for it a wait for the row loads too)
    typedef __attribute__((address_space(3))) uint32_t lds_u32;
    const lds_u32 *const L = (const lds_u32 *)lds;
    auto locate = [&](uint32_t g) -> RowRef {
        uint32_t r = g, j = 0;
        if (!simple) {
            uint32_t lo = 0, hi = n_reqs;
            while (hi - lo > 1u) {
                const uint32_t mid = (lo + hi) >> 1;
                if (L[m.pref + mid] <= g) lo = mid; else hi = mid;
            }
            r = lo;
            j = g - L[m.pref + r];
        }
        RowRef ref;
        if (!a.paged) {
            int64_t row;
            if (index_mode) {
                row = (int64_t)a.row_index[simple ? g : L[m.pref_all + r] + j];
            } else if (a.table_in_lds) {
                row = (int64_t)L[m.rb + r] + (int64_t)j * (int64_t)L[m.tab + 4u * r + 2u];
            } else {
                row = (int64_t)a.row0[r];
                if (j) row += (int64_t)j * (int64_t)a.req_table[r].z;
            }
            ref.ok = row >= 0 && row < a.n_src_rows;
            ref.base = src + (ref.ok ? row : 0) * a.row_stride_b;
        } else {
            uint32_t tok0, tstep, seq_row;
            if (a.table_in_lds) {
                tok0 = L[m.tab + 4u * r + 1u]; tstep = L[m.tab + 4u * r + 2u]; seq_row = L[m.rb + r];
            } else {
                const uint4 e = a.req_table[r];
                tok0 = e.y; tstep = e.z; seq_row = a.row0[r];
            }
            const uint32_t t = tok0 + j * tstep;            // host keeps token positions below 2^31
            const uint32_t lb = a.bs_shift < 32u ? t >> a.bs_shift : t / a.block_size;
            const uint32_t slot = t - lb * a.block_size;
            const int64_t blk = (int64_t)a.block_table[(int64_t)seq_row * a.bt_stride + (int64_t)lb];
            ref.ok = blk >= 0 && blk < a.n_src_rows;
            ref.base = src + (ref.ok ? blk : 0) * a.block_stride_b + (int64_t)slot * a.slot_stride_b;
        }
        return ref;
    };
    auto unit_ptr = [&](const RowRef &ref, uint32_t c) -> const uint8_t * {
        if (!a.paged) return ref.base + (uint64_t)c * NB_IN;
        const uint32_t seg = a.seg_shift < 32u ? c >> a.seg_shift : c / a.seg_units;
        const uint32_t cc = c - seg * a.seg_units;
        return ref.base + (int64_t)L[m.heads + seg] * a.head_stride_b + (uint64_t)cc * NB_IN;
    };
    // Loads are never put under a condition of their own: the compiler then waits for each
    // one before it issues the next (a register copy where the branches join), and four
    // loads in flight become four trips to memory.  A unit that is not wanted (past the
    // end, or of a row whose index left the source) is read from the control block instead
    // and replaced by zeros, or skipped, when it is stored.
    const uint8_t *const safe_src = reinterpret_cast<const uint8_t *>(a.ctrl);
    auto load_unit = [&](const RowRef &ref, uint32_t c, bool want) -> unit_t {
        const uint8_t *p = want ? unit_ptr(ref, want ? c : 0u) : safe_src;
        // both are device memory; said explicitly, or the choice between two pointers costs the load its type
        typedef __attribute__((address_space(1))) const unit_t global_unit_t;
        return *(global_unit_t *)p;
    };
    auto zero_unless = [](bool keep, unit_t v) -> unit_t { return keep ? v : unit_t{}; };

    if (!dropped) {
        // ---- header, request table and all pad bytes: workgroup 0.  The header is put
        //      together in LDS and leaves as four 16-byte stores.
        if (blockIdx.x == 0) {
            if (tid == 0) {
                uint32_t *h = lds + m.hdr;
                h[0] = 0x32494D44u;
                h[1] = 1u | (64u << 16);
                const uint64_t seq_y = ((uint64_t)lds[m.bcast + 8] | ((uint64_t)lds[m.bcast + 9] << 32)) + y;
                h[2] = (uint32_t)seq_y;          h[3] = (uint32_t)(seq_y >> 32);
                h[4] = lds[m.bcast + 10];        h[5] = lds[m.bcast + 11];      // step id
                h[6] = point_id;
                h[7] = a.src_dtype | (a.out_dtype << 8) | (a.summary_mask << 16) | (a.rec_flags << 24);
                h[8] = n_reqs;  h[9] = n_rows;  h[10] = a.row_elems;  h[11] = a.rank_tag;
                h[12] = (uint32_t)record_bytes;  h[13] = (uint32_t)(record_bytes >> 32);
                h[14] = (uint32_t)payload_bytes; h[15] = (uint32_t)(payload_bytes >> 32);
            }
            lds_barrier();
            if (tid < 4) {
                const uint32_t *h = lds + m.hdr + 4 * tid;
                u32x4 v = {h[0], h[1], h[2], h[3]};
                ring_store<u32x4>(w, 16u * tid, v);
            }
            const uint32_t tab_slots = (uint32_t)(table_bytes / 16u);
            for (uint32_t r = tid; r < tab_slots; r += kThreads) {
                u32x4 v = {0u, 0u, 0u, 0u};
                if (r < n_reqs) {
                    uint4 e;
                    if (a.table_in_lds) e = ltab[r];
                    else { e = a.req_table[r]; if (!simple) e.w = pref[r + 1] - pref[r]; }
                    v.x = e.x; v.y = e.y; v.z = e.z; v.w = e.w;
                }
                ring_store<u32x4>(w, 64u + 16ull * r, v);
            }
            {
                const uint32_t pad = (uint32_t)(off_sum - off_payload - payload_bytes);
                if (tid < pad) ring_store<uint8_t>(w, off_payload + payload_bytes + tid, (uint8_t)0);
                const uint32_t spad = (uint32_t)(sum_arr - (uint64_t)n_rows * 4u) / 4u;
                for (uint32_t k = tid; k < n_sum * spad; k += kThreads) {
                    const uint32_t arr = k / spad, i = k - arr * spad;
                    ring_store<uint32_t>(w, off_sum + arr * sum_arr + (uint64_t)n_rows * 4u + 4ull * i, 0u);
                }
            }
        }

        if constexpr (!SUMM) {
            if constexpr (OUT != OUT_NONE) {
                Accum dummy = {0.f, 0.f, 0u};
                if (a.units_per_row >= kThreads) {
                    // ---- long rows: a work item is 1024 consecutive units: a quarter or more of one
                    //      row, or 2 / 4 whole rows of 512 / 256 units; rows are located once per
                    //      item, not per unit.  Software pipelined: the next item's 4 loads per lane
                    //      are in flight while this one is converted and stored.
                    const uint32_t rpi = (a.units_per_row < CH && CH % a.units_per_row == 0u)
                                             ? CH / a.units_per_row : 1u;          // rows per item
                    const uint64_t n_items = rpi > 1u ? ((uint64_t)n_rows + rpi - 1u) / rpi
                                                      : (uint64_t)n_rows * cpr;
                    // unit k of this lane in item `it`: its flat position in the payload, loaded value
                    auto fetch = [&](uint64_t it, unit_t (&v)[U], uint64_t (&pos)[U], bool (&live)[U], uint32_t &okm) {
                        RowRef ref = {nullptr, 0}, refs[U];
                        uint32_t g_prev = 0xFFFFFFFFu, cs[U];
                        okm = 0;
                        // first where every unit comes from (a row's place may take a load of its own to
                        // find), then all the unit loads together
#pragma unroll
                        for (uint32_t k = 0; k < U; k++) {
                            uint32_t g, c;
                            if (rpi > 1u) {
                                const uint32_t idx = k * kThreads + tid;
                                const uint32_t rk = idx >> a.upr_shift;        // units_per_row is 256 or 512
                                g = (uint32_t)it * rpi + rk;
                                c = idx - (rk << a.upr_shift);
                            } else {
                                g = cpr == 1u ? (uint32_t)it : (uint32_t)(it / cpr);
                                c = (uint32_t)(it - (uint64_t)g * cpr) * CH + k * kThreads + tid;
                            }
                            live[k] = g < n_rows && c < a.units_per_row;
                            pos[k] = (uint64_t)g * a.units_per_row + c;
                            if (live[k] && g != g_prev) {
                                ref = locate(g);
                                g_prev = g;
                                if (!ref.ok && c == 0) atomicAdd((unsigned long long *)&a.ctrl->bad_rows, 1ull);
                            }
                            refs[k] = ref;
                            cs[k] = c;
                        }
                        asm volatile("" ::: "memory");      // keep the two phases apart
#pragma unroll
                        for (uint32_t k = 0; k < U; k++) {
                            const bool want = live[k] && refs[k].ok != 0;
                            okm |= want ? 1u << k : 0u;
                            v[k] = load_unit(refs[k], cs[k], want);
                        }
                    };
                    uint64_t it = blockIdx.x;
                    if (it < n_items) {
                        unit_t v[U];
                        uint64_t pos[U];
                        bool live[U];
                        uint32_t okm = 0;
                        if (pre) {      // decode-shaped, rows of >= 1024 units handled one per item
                            const uint32_t g = cpr == 1u ? (uint32_t)it : (uint32_t)(it / cpr);
                            const uint32_t c0 = (uint32_t)(it - (uint64_t)g * cpr) * CH + tid;
#pragma unroll
                            for (uint32_t k = 0; k < U; k++) {
                                const uint32_t c = c0 + k * kThreads;
                                v[k] = pre_v[k];
                                live[k] = c < a.units_per_row;
                                okm |= live[k] && pre_ref.ok ? 1u << k : 0u;
                                pos[k] = (uint64_t)g * a.units_per_row + c;
                            }
                            if (!pre_ref.ok && c0 == 0) atomicAdd((unsigned long long *)&a.ctrl->bad_rows, 1ull);
                        } else {
                            fetch(it, v, pos, live, okm);
                        }
                        for (;;) {
                            const uint64_t nxt = it + gridDim.x;
                            const bool more = nxt < n_items;
                            unit_t v_n[U];
                            uint64_t pos_n[U];
                            bool live_n[U];
                            uint32_t okm_n = 0;
                            if (more) fetch(nxt, v_n, pos_n, live_n, okm_n);
#pragma unroll
                            for (uint32_t k = 0; k < U; k++)
                                if (live[k])
                                    emit_unit<ES_IN, VEC, OUT, false>(w, off_payload + pos[k] * NB_OUT,
                                                                      zero_unless((okm >> k) & 1u, v[k]), a.src_dtype, dummy);
                            if (!more) break;
                            it = nxt;
                            okm = okm_n;
#pragma unroll
                            for (uint32_t k = 0; k < U; k++) { v[k] = v_n[k]; pos[k] = pos_n[k]; live[k] = live_n[k]; }
                        }
                    }
                } else {
                    // ---- short rows: the n_rows x units_per_row units are dealt to lanes in order,
                    //      so stores stay fully coalesced; 4 loads in flight per lane.
                    //      A wavefront's 64 units of one slice lie in at most 64/upr + 2 rows.  When
                    //      the rows of its four slices fit the 64 lanes, each lane locates one row
                    //      (all of them in a single pass) and every unit picks up its row's place by
                    //      shuffle: locating a row costs on the order of a hundred instructions, and
                    //      done per unit that, not memory, is what the launch spends its time on.
                    const uint32_t total = (uint32_t)((uint64_t)n_rows * a.units_per_row);  // host keeps it below 2^32
                    const uint32_t upr = a.units_per_row;
                    auto row_of = [&](uint32_t u) { return a.upr_shift < 32u ? u >> a.upr_shift : u / upr; };
                    const bool shared_locate = 64u / upr + 2u <= 16u;
                    const uint32_t slice_stride = gridDim.x * kThreads;
                    for (uint64_t t0 = (uint64_t)blockIdx.x * kThreads; t0 < total; t0 += (uint64_t)slice_stride * U) {
                        unit_t v[U];
                        bool live[U], okk[U];
                        uint32_t my_lo = 0, my_hi = 0, my_ok = 0, my_first = 0;
                        if (shared_locate) {
                            const uint32_t sl = lane >> 4, j = lane & 15u;
                            const uint64_t us = t0 + (uint64_t)sl * slice_stride + wave * 64u;
                            if (us < total) {
                                const uint32_t ue = us + 63u < total ? (uint32_t)us + 63u : total - 1u;
                                my_first = row_of((uint32_t)us);
                                const uint32_t g = my_first + j;
                                if (g <= row_of(ue)) {
                                    const RowRef ref = locate(g);
                                    my_lo = (uint32_t)(uintptr_t)ref.base;
                                    my_hi = (uint32_t)((uintptr_t)ref.base >> 32);
                                    my_ok = ref.ok ? 1u : 0u;
                                    // a bad row is counted where its first unit lies
                                    const uint64_t fu = (uint64_t)g * upr;
                                    if (!ref.ok && fu >= us && fu <= ue)
                                        atomicAdd((unsigned long long *)&a.ctrl->bad_rows, 1ull);
                                }
                            }
                        }
#pragma unroll
                        for (uint32_t k = 0; k < U; k++) {
                            const uint64_t u = t0 + (uint64_t)k * slice_stride + tid;
                            live[k] = u < total;
                            const uint32_t u32 = live[k] ? (uint32_t)u : total - 1u;
                            const uint32_t g = row_of(u32);
                            const uint32_t c = u32 - g * upr;
                            RowRef ref;
                            if (shared_locate) {
                                // executed by all 64 lanes: a shuffle reads nothing useful from a lane that is off
                                const uint32_t first_k = __shfl(my_first, (int)(k << 4), 64);
                                const int src = (int)(((k << 4) + (g - first_k)) & 63u);
                                const uint32_t lo = __shfl(my_lo, src, 64), hi = __shfl(my_hi, src, 64);
                                ref.ok = __shfl(my_ok, src, 64);
                                ref.base = reinterpret_cast<const uint8_t *>(((uint64_t)hi << 32) | lo);
                                if (!live[k]) ref.ok = 0;
                            } else {
                                ref.base = nullptr;
                                ref.ok = 0;
                                if (live[k]) {
                                    ref = locate(g);
                                    if (!ref.ok && c == 0) atomicAdd((unsigned long long *)&a.ctrl->bad_rows, 1ull);
                                }
                            }
                            okk[k] = live[k] && ref.ok != 0;
                            v[k] = load_unit(ref, c, okk[k]);
                        }
#pragma unroll
                        for (uint32_t k = 0; k < U; k++) {
                            const uint64_t u = t0 + (uint64_t)k * slice_stride + tid;
                            if (live[k])
                                emit_unit<ES_IN, VEC, OUT, false>(w, off_payload + u * NB_OUT, zero_unless(okk[k], v[k]),
                                                                  a.src_dtype, dummy);
                        }
                    }
                }
            }
        } else {
            // ---- row-wise pass with summaries: a workgroup (or a wavefront) per row.  A step is
            //      4 units per lane of one row; rows longer than that take several steps.  Steps
            //      are software pipelined (the next step's loads are issued before this step is
            //      converted, stored and accumulated), across row boundaries too.
            float *red = reinterpret_cast<float *>(lds + m.red);
            const uint32_t spr = (a.units_per_row + gsz * U - 1u) / (gsz * U);     // steps per row
            const uint64_t row_stride_g = (uint64_t)gridDim.x * rpw;
            // a step = (g0: first row of the workgroup's current group, pass)
            auto fetch = [&](uint64_t st_g0, uint32_t st_pass, RowRef &ref, unit_t (&v)[U]) {
                const uint64_t g = st_g0 + sub;
                const bool row_live = g < n_rows;
                if (row_live && st_pass == 0) {
                    ref = locate((uint32_t)g);
                    if (!ref.ok && l == 0) atomicAdd((unsigned long long *)&a.ctrl->bad_rows, 1ull);
                }
#pragma unroll
                for (uint32_t k = 0; k < U; k++) {
                    const uint32_t c = l + (st_pass * U + k) * gsz;
                    v[k] = load_unit(ref, c, row_live && ref.ok != 0 && c < a.units_per_row);
                }
            };
            uint64_t cur_g0 = (uint64_t)blockIdx.x * rpw;
            uint32_t cur_pass = 0;
            if (cur_g0 < n_rows) {
                RowRef ref = {nullptr, 0};
                unit_t v[U];
                if (pre) {
                    ref = pre_ref;
#pragma unroll
                    for (uint32_t k = 0; k < U; k++) v[k] = pre_v[k];
                    // (fetch() counts the rows it locates; this one was located up front)
                    if (!ref.ok && l == 0 && cur_g0 + sub < n_rows) atomicAdd((unsigned long long *)&a.ctrl->bad_rows, 1ull);
                } else {
                    fetch(cur_g0, cur_pass, ref, v);
                }
                Accum acc = {0.f, 0.f, 0u};
                for (;;) {
                    uint64_t nxt_g0 = cur_g0;
                    uint32_t nxt_pass = cur_pass + 1u;
                    if (nxt_pass == spr) { nxt_pass = 0; nxt_g0 += row_stride_g; }
                    const bool more = nxt_g0 < n_rows;
                    RowRef ref_n = ref;             // a later pass of the same row keeps the row
                    unit_t v_n[U];
                    if (more) fetch(nxt_g0, nxt_pass, ref_n, v_n);
                    const uint64_t g = cur_g0 + sub;
                    const bool active = g < n_rows;
                    if (active) {
                        const uint64_t row_off = off_payload + g * a.units_per_row * NB_OUT;
#pragma unroll
                        for (uint32_t k = 0; k < U; k++) {
                            const uint32_t c = l + (cur_pass * U + k) * gsz;
                            if (c < a.units_per_row)
                                emit_unit<ES_IN, VEC, OUT, true>(w, row_off + (uint64_t)c * NB_OUT,
                                                                 zero_unless(ref.ok != 0, v[k]), a.src_dtype, acc);
                        }
                    }
                    if (cur_pass == spr - 1u) {     // the row is complete: reduce and store its summaries
                        acc.ss = wave_sum(acc.ss);
                        acc.s = wave_sum(acc.s);
                        uint32_t am = wave_max_u32(fold_am<ES_IN, VEC>(acc.am));
                        if (rpw == 1u) {
                            lds_barrier();        // the previous row's readers are done with red[]
                            if (lane == 0) {
                                red[wave] = acc.ss;
                                red[4 + wave] = acc.s;
                                reinterpret_cast<uint32_t *>(red)[8 + wave] = am;
                            }
                            lds_barrier();
                            acc.ss = (red[0] + red[1]) + (red[2] + red[3]);
                            acc.s = (red[4] + red[5]) + (red[6] + red[7]);
                            const uint32_t *ra = reinterpret_cast<const uint32_t *>(red) + 8;
                            const uint32_t m01 = ra[0] > ra[1] ? ra[0] : ra[1], m23 = ra[2] > ra[3] ? ra[2] : ra[3];
                            am = m01 > m23 ? m01 : m23;
                        }
                        if (active && l == 0) {
                            uint64_t o = off_sum + g * 4u;
                            if (a.summary_mask & 1u) { ring_store<float>(w, o, sqrtf(acc.ss)); o += sum_arr; }
                            if (a.summary_mask & 2u) { ring_store<float>(w, o, acc.s / (float)a.row_elems); o += sum_arr; }
                            if (a.summary_mask & 4u) { ring_store<float>(w, o, am_value(am, a.src_dtype)); }
                        }
                        acc = Accum{0.f, 0.f, 0u};
                    }
                    if (!more) break;
                    cur_g0 = nxt_g0;
                    cur_pass = nxt_pass;
                    ref = ref_n;
#pragma unroll
                    for (uint32_t k = 0; k < U; k++) v[k] = v_n[k];
                }
            }
        }
    }
}


// ---------------------------------------------------------------- decode-shaped capture
// The common case of the paper's workloads (every layer's hidden state at a decode step):
// bf16 rows, one per request, no keep mask.  Everything about the record except its place
// in the ring is known on the host, so the kernel is straight-line: a workgroup per row
// issues its loads at once, an extra workgroup writes header, table and pads and publishes.
// A small capture is bound by instructions issued and dependent memory trips, not by
// bytes; the general kernel above executes several times as many instructions per row.
// Kernel arguments of the decode-shaped kernel.  The scalar cache is cold at every launch,
// so each 64-byte line of the argument block costs a trip to memory when it is first
// touched, and the compiler, left alone, puts each argument load next to its first use:
// a chain of such trips, one after another, that is longer than the copy itself.  What
// every workgroup needs therefore sits in the first two lines, what only the extra
// workgroup needs in the third, and all three are fetched together at the top.
struct DecodeArgs {
    // line 0
    uint64_t spare0;
    int64_t row_stride_b;
    const int32_t *rows;            // row per request (int32 indices or uint32 first rows), unless consecutive
    uint8_t *ring;
    uint64_t cap;
    DevCtrl *ctrl;
    const StepParams *step;
    uint64_t tail_floor;
    // line 1
    uint64_t record_bytes, off_payload, off_sum, sum_arr;
    uint32_t n_src_rows, n_reqs, units_per_row, row_first;
    uint32_t flags;                 // kDec*
    uint32_t node, summary_mask, row_elems;
    // line 2
    uint64_t seq, step_id;
    const uint4 *req_table;
    CommitSlot *cslot;
    uint64_t payload_bytes;
    uint32_t spare1, hdr7, rank_tag, pad;
    const uint64_t *tail_src;       // where the extra workgroup reads the drained-up-to mark (may be NULL)
    // line 3
    const uint8_t *keep_mask;       // keep vector (MASK variants): request r is captured iff keep_mask[r] != 0
    uint32_t n_wg_rows;             // row workgroups = rows listed (= n_reqs unless requests list several rows)
    uint32_t spare32;
    uint64_t spare[6];
};
static_assert(sizeof(DecodeArgs) == 256, "four lines");
constexpr uint32_t kDecDropNewest = 1u, kDecConsecutive = 2u, kDecIndexed = 4u, kDecParIn = 8u;

// MASK: the paper's best-effort path (section 4.4): a batch-aligned keep vector, read when the
// kernel runs, decides per request.  Every workgroup reads the whole vector (at most 1024
// bytes) together with its other loads, the wavefronts ballot it into 16 words of LDS, and
// each workgroup derives from those the record's row count and its own row's place.  The
// row itself is loaded before the vector is known and thrown away if the request is out.
template <int OUT, bool SUMM, bool MASK>
__global__ void __launch_bounds__(kThreads) capture_decode_kernel(const DecodeArgs a, const BatchArgs b)
{
    __shared__ uint32_t sh[32];
    __shared__ uint64_t kept_bits[16];      // MASK: bit i of word q = request 64 q + i is kept
    const uint32_t y = blockIdx.y;          // which tensor of the batch
    const uint8_t *const src = b.src[y];
    const uint32_t point_id = b.point[y];
    touch_argument_lines(a, src, point_id);
    constexpr uint32_t U = 4;
    constexpr uint32_t NB_OUT = out_unit_bytes<2, 8, OUT>();
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t par = (a.flags & kDecParIn) ? 1u : 0u;
    const bool meta_wg = blockIdx.x == a.n_wg_rows;
    constexpr uint32_t kCtlTid = kThreads - 64u;

    // control words first (they depend on nothing but the arguments), then the row
    uint64_t cnt_cap[3] = {0, 0, 0}, cnt_drop[3] = {0, 0, 0}, tail_now = 0, seq = a.seq;
    RawControl raw = {};
    if (tid == kCtlTid) raw = fetch_control(a.ctrl, par, a.step);
    uint32_t kb[4] = {0u, 0u, 0u, 0u};
    if constexpr (MASK) {
#pragma unroll
        for (uint32_t k = 0; k < 4; k++) {
            const uint32_t r = tid + k * kThreads;
            kb[k] = a.keep_mask[r < a.n_reqs ? r : 0u];
        }
    }
    u32x4 v[U];
    bool ok = false;
    if (!meta_wg) {
        const uint32_t g = blockIdx.x;
        // the usual decode layout (request i in row first + i) saves the dependent trip to the table
        const int64_t row = (a.flags & kDecConsecutive) ? (int64_t)a.row_first + g
                            : (a.flags & kDecIndexed) ? (int64_t)a.rows[g]
                                                      : (int64_t)reinterpret_cast<const uint32_t *>(a.rows)[g];
        ok = row >= 0 && row < (int64_t)a.n_src_rows;
        const uint8_t *base = src + (ok ? row : 0) * a.row_stride_b;
#pragma unroll
        for (uint32_t k = 0; k < U; k++) v[k] = u32x4{0u, 0u, 0u, 0u};
        if (ok) {
            // straight-line loads: lanes past the end of the row fetch its first unit again and
            // ignore it (a load under its own condition makes the compiler wait between loads)
#pragma unroll
            for (uint32_t k = 0; k < U; k++) {
                const uint32_t c = tid + k * kThreads;
                v[k] = *reinterpret_cast<const u32x4 *>(base + (uint64_t)(c < a.units_per_row ? c : 0u) * 16u);
            }
        }
    }
    if constexpr (MASK) {
#pragma unroll
        for (uint32_t k = 0; k < 4; k++) {
            const uint32_t r = tid + k * kThreads;
            const uint64_t b = __ballot(r < a.n_reqs && kb[k] != 0u);
            if (lane == 0) kept_bits[k * 4u + wave] = b;
        }
    }
    if (tid == kCtlTid) {
        // the drained-up-to mark for the next launch's drop decision, read where the host keeps
        // it by the extra workgroup's lane, after every other load of that lane
        const uint64_t *ts = meta_wg && y == 0 && a.tail_src ? a.tail_src : &a.ctrl->tail;
        tail_now = ld_system(ts);
        const Control ct = resolve_control(raw, a.step != nullptr, a.node, a.tail_floor, a.seq, a.step_id,
                                           a.flags & kDecDropNewest);
        seq = ct.seq;
        for (int i = 0; i < 3; i++) { cnt_cap[i] = raw.cap[i]; cnt_drop[i] = raw.drop[i]; }
        const uint64_t base = ct.head % a.cap;
        sh[0] = (uint32_t)ct.head;  sh[1] = (uint32_t)(ct.head >> 32);
        sh[2] = (uint32_t)ct.tail;  sh[3] = (uint32_t)(ct.tail >> 32);
        sh[4] = (uint32_t)base;     sh[5] = (uint32_t)(base >> 32);
        sh[6] = ct.flags;
        sh[24] = (uint32_t)ct.seq;      sh[25] = (uint32_t)(ct.seq >> 32);
        sh[26] = (uint32_t)ct.step_id;  sh[27] = (uint32_t)(ct.step_id >> 32);
    }
    // Summaries are taken before the one barrier of this kernel, which then hands over both
    // the control words and the wavefronts' partial sums: the rows arrive later than the
    // control words anyway, and a second barrier behind the stores would put the summary
    // stores a good half microsecond behind the row stores.
    if constexpr (SUMM) {
        Accum acc = {0.f, 0.f, 0u};
        if (!meta_wg) {
#pragma unroll
            for (uint32_t k = 0; k < U; k++) {
                const uint32_t c = tid + k * kThreads;
                if (c < a.units_per_row) emit_unit<2, 8, OUT_NONE, true>(RingW{}, 0, v[k], a.hdr7 & 0xFFu, acc);
            }
            acc.ss = wave_sum(acc.ss);
            acc.s = wave_sum(acc.s);
            const uint32_t am = wave_max_u32(fold_am<2, 8>(acc.am));
            float *red = reinterpret_cast<float *>(sh + 8);
            if (lane == 0) {
                red[wave] = acc.ss;
                red[4 + wave] = acc.s;
                sh[16 + wave] = am;
            }
        }
    }
    lds_barrier();
    const uint64_t head0 = (uint64_t)sh[0] | ((uint64_t)sh[1] << 32);
    const uint64_t tail = (uint64_t)sh[2] | ((uint64_t)sh[3] << 32);
    const uint32_t flags = sh[6];
    const bool publisher = meta_wg && y == 0 && tid == kCtlTid;
    if (flags & kStepSkip) {    // sampled-out replay: pass head and tail on, capture nothing
        if (publisher) {
            a.ctrl->head[par ^ 1u] = head0;
            a.ctrl->tail_for[par ^ 1u] = tail_now > raw.tail_for ? tail_now : raw.tail_for;
        }
        return;
    }
    // record geometry: known on the host, or from the keep vector
    uint32_t n_rows = a.n_wg_rows, my_row = blockIdx.x;
    bool kept = true;
    uint64_t record_bytes = a.record_bytes, payload_bytes = a.payload_bytes, off_sum = a.off_sum, sum_arr = a.sum_arr;
    if constexpr (MASK) {
        const uint32_t q_me = blockIdx.x >> 6;
        n_rows = 0;
        my_row = 0;
#pragma unroll
        for (uint32_t q = 0; q < 16; q++) {
            const uint32_t pc = (uint32_t)__popcll(kept_bits[q]);
            n_rows += pc;
            if (q < q_me) my_row += pc;
        }
        if (!meta_wg) {
            const uint64_t mine = kept_bits[q_me & 15u], bit = 1ull << (blockIdx.x & 63u);
            kept = (mine & bit) != 0;
            my_row += (uint32_t)__popcll(mine & (bit - 1u));
        }
        payload_bytes = (uint64_t)n_rows * a.units_per_row * NB_OUT;
        off_sum = a.off_payload + ((payload_bytes + 63u) & ~63ull);
        sum_arr = ((uint64_t)n_rows * 4u + 63u) & ~63ull;
        record_bytes = off_sum + (uint64_t)__popc(a.summary_mask & 7u) * sum_arr;
    }
    // record y of the launch lies y records behind the head the launch found (all records of a
    // batch have one size: record y fits iff the y before it did, and then they were kept)
    const bool drop_newest = (flags & kStepDropNewest) != 0;
    const uint64_t head = head0 + (uint64_t)y * record_bytes;
    const bool dropped = drop_newest && head - tail + record_bytes > a.cap;
    RingW w;
    w.ring = a.ring;
    w.cap = a.cap;
    w.base = ((uint64_t)sh[4] | ((uint64_t)sh[5] << 32)) + (uint64_t)y * record_bytes;
    if (w.base >= w.cap) w.base -= w.cap;   // the issuer made sure a launch's records fit the ring together

    if (meta_wg) {
        if (publisher) {
            DevCtrl *c = a.ctrl;
            const uint64_t nb_rec = gridDim.y;
            uint64_t n_fit = nb_rec;
            if (drop_newest) {
                const uint64_t used = head0 - tail;
                n_fit = used < a.cap ? (a.cap - used) / record_bytes : 0u;
                n_fit = n_fit < nb_rec ? n_fit : nb_rec;
            }
            const uint64_t n_drop = nb_rec - n_fit;
            const uint64_t new_head = head0 + n_fit * record_bytes;
            if (n_drop) {
                cnt_drop[0] += n_drop; cnt_drop[1] += n_drop * n_rows; cnt_drop[2] += n_drop * record_bytes;
                c->dropped_records = cnt_drop[0]; c->dropped_rows = cnt_drop[1]; c->dropped_bytes = cnt_drop[2];
            }
            if (n_fit) {
                cnt_cap[0] += n_fit; cnt_cap[1] += n_fit * n_rows; cnt_cap[2] += n_fit * record_bytes;
                c->captured_records = cnt_cap[0]; c->captured_rows = cnt_cap[1]; c->captured_bytes = cnt_cap[2];
            }
            c->head[par ^ 1u] = new_head;
            c->tail_for[par ^ 1u] = tail_now > raw.tail_for ? tail_now : raw.tail_for;
            const uint64_t last_seq = seq + nb_rec - 1u;
            CommitSlot *h = a.step ? &c->slots[last_seq % kCommitSlots] : a.cslot;
            h->head = new_head;
            h->captured_records = cnt_cap[0]; h->captured_rows = cnt_cap[1]; h->captured_bytes = cnt_cap[2];
            h->dropped_records = cnt_drop[0]; h->dropped_rows = cnt_drop[1]; h->dropped_bytes = cnt_drop[2];
            h->seq_plus1 = last_seq + 1u;
        }
        if (dropped && tid == kCtlTid) atomicAdd(&a.ctrl->point_drops[point_id & 4095u], 1u);
        if (dropped) return;
        if (tid < 4) {
            u32x4 hv;
            const uint64_t seq_y = ((uint64_t)sh[24] | ((uint64_t)sh[25] << 32)) + y;
            if (tid == 0) hv = u32x4{0x32494D44u, 1u | (64u << 16), (uint32_t)seq_y, (uint32_t)(seq_y >> 32)};
            else if (tid == 1) hv = u32x4{sh[26], sh[27], point_id, a.hdr7};
            else if (tid == 2) hv = u32x4{a.n_reqs, n_rows, a.row_elems, a.rank_tag};
            else hv = u32x4{(uint32_t)record_bytes, (uint32_t)(record_bytes >> 32), (uint32_t)payload_bytes,
                            (uint32_t)(payload_bytes >> 32)};
            ring_store<u32x4>(w, 16u * tid, hv);
        }
        const uint32_t tab_slots = (uint32_t)((a.off_payload - 64u) / 16u);
        for (uint32_t r = tid; r < tab_slots; r += kThreads) {
            u32x4 tv = {0u, 0u, 0u, 0u};
            if (r < a.n_reqs) {
                const uint4 e = a.req_table[r];
                tv.x = e.x; tv.y = e.y; tv.z = e.z; tv.w = e.w;
                if constexpr (MASK) tv.w = (uint32_t)((kept_bits[(r >> 6) & 15u] >> (r & 63u)) & 1ull);
            }
            ring_store<u32x4>(w, 64u + 16ull * r, tv);
        }
        const uint32_t pad = (uint32_t)(off_sum - a.off_payload - payload_bytes);
        if (tid < pad) ring_store<uint8_t>(w, a.off_payload + payload_bytes + tid, (uint8_t)0);
        const uint32_t n_sum = __popc(a.summary_mask & 7u);
        const uint32_t spad = (uint32_t)(sum_arr - (uint64_t)n_rows * 4u) / 4u;
        for (uint32_t k = tid; k < n_sum * spad; k += kThreads) {
            const uint32_t arr = k / spad, i = k - arr * spad;
            ring_store<uint32_t>(w, off_sum + arr * sum_arr + (uint64_t)n_rows * 4u + 4ull * i, 0u);
        }
        return;
    }

    if (dropped || !kept) return;
    const uint32_t g = my_row;
    if (!ok && tid == 0) atomicAdd((unsigned long long *)&a.ctrl->bad_rows, 1ull);
    Accum acc = {0.f, 0.f, 0u};
    const uint64_t row_off = a.off_payload + (uint64_t)g * a.units_per_row * NB_OUT;
#pragma unroll
    for (uint32_t k = 0; k < U; k++) {
        const uint32_t c = tid + k * kThreads;
        if (c < a.units_per_row)
            emit_unit<2, 8, OUT, false>(w, row_off + (uint64_t)c * NB_OUT, v[k], a.hdr7 & 0xFFu, acc);
    }
    if constexpr (SUMM) {
        if (tid == 0) {
            const float *red = reinterpret_cast<const float *>(sh + 8);
            const float ss = (red[0] + red[1]) + (red[2] + red[3]);
            const float sm = (red[4] + red[5]) + (red[6] + red[7]);
            const uint32_t m01 = sh[16] > sh[17] ? sh[16] : sh[17], m23 = sh[18] > sh[19] ? sh[18] : sh[19];
            const uint32_t am = m01 > m23 ? m01 : m23;
            uint64_t o = off_sum + (uint64_t)g * 4u;
            if (a.summary_mask & 1u) { ring_store<float>(w, o, sqrtf(ss)); o += sum_arr; }
            if (a.summary_mask & 2u) { ring_store<float>(w, o, sm / (float)a.row_elems); o += sum_arr; }
            if (a.summary_mask & 4u) { ring_store<float>(w, o, am_value(am, a.hdr7 & 0xFFu)); }
        }
    }
}

// ---------------------------------------------------------------- small kernels
struct UploadChunk {
    uint32_t w[896];
};

__global__ void __launch_bounds__(kThreads) upload_kernel(uint32_t *dst, const UploadChunk c, uint32_t n)
{
    for (uint32_t i = threadIdx.x; i < n; i += kThreads) dst[i] = c.w[i];
}

// Start of a replayable step (an ordinary launch in front of the graph's): the step's
// parameter block, and head / tail_for carried over to the copy its first launch reads.
__global__ void step_begin_kernel(DevCtrl *ctrl, StepParams *step, const StepParams v, uint32_t par_from,
                                  uint32_t par_to, const uint64_t *host_tail)
{
    if (threadIdx.x != 0) return;
    *step = v;
    if (host_tail) ctrl->tail = ld_system(host_tail);    // the step's launches read this copy
    if (par_from != par_to) {
        ctrl->head[par_to] = ctrl->head[par_from];
        ctrl->tail_for[par_to] = ctrl->tail_for[par_from];
    }
}

// Put a control block back to "empty stream, nothing counted": the chain words and the running
// counters (a fill kernel, so that a caller under graph capture records a kernel node).
__global__ void ctrl_reset_kernel(DevCtrl *ctrl)
{
    if (threadIdx.x != 0) return;
    ctrl->head[0] = ctrl->head[1] = 0;
    ctrl->tail_for[0] = ctrl->tail_for[1] = 0;
    ctrl->tail = 0;
    ctrl->captured_records = ctrl->captured_rows = ctrl->captured_bytes = 0;
    ctrl->dropped_records = ctrl->dropped_rows = ctrl->dropped_bytes = 0;
    ctrl->bad_rows = 0;
}

// Fetch one commit slot into pinned host memory: a small launch of its own on the producer's
// stream, so the capture kernel itself never writes across PCIe (such a store is
// acknowledged only after some 4-5 microseconds, and a kernel cannot retire before its
// stores have been).
__global__ void fetch_slot_kernel(const CommitSlot *src, CommitSlot *dst_host)
{
    const uint32_t i = threadIdx.x;
    if (i < sizeof(CommitSlot) / 8u)
        reinterpret_cast<volatile uint64_t *>(dst_host)[i] = reinterpret_cast<const uint64_t *>(src)[i];
}

// Drain by kernel: 16-byte loads from the device ring, 16-byte stores into the pinned
// host ring (posted PCIe writes).
__global__ void __launch_bounds__(kThreads) drain_kernel(const uint8_t *ring, uint64_t cap, uint8_t *host,
                                                         uint64_t host_cap, uint64_t from, uint64_t nbytes)
{
    const uint64_t n_units = nbytes / 16u;
    const uint64_t s0 = from % cap, d0 = from % host_cap;
    for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < n_units;
         i += (uint64_t)gridDim.x * kThreads) {
        uint64_t s = s0 + i * 16u, d = d0 + i * 16u;
        if (s >= cap) s -= cap;
        if (d >= host_cap) d -= host_cap;
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(ring + s));
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(host + d));
    }
}

// ---------------------------------------------------------------- launchers
// A benchmark may ask for the next capture launch of its thread to be timed by the hardware itself:
// the two events then take the dispatch's own start and end time stamps (what a profiler reports
// as the kernel's duration), not the times at which markers around the launch were reached.
static thread_local hipEvent_t t_time_start = nullptr, t_time_stop = nullptr;

extern "C" dmi_status_t dmi_debug_time_next_launch(void *start_event, void *stop_event)
{
    t_time_start = static_cast<hipEvent_t>(start_event);
    t_time_stop = static_cast<hipEvent_t>(stop_event);
    return DMI_OK;
}

#define DMI_LAUNCH_CAPTURE(in_step, kernel, grid, lds, stream, ...)                                                   \
    do {                                                                                                              \
        if (t_time_start && t_time_stop && !(in_step)) {                                                              \
            hipExtLaunchKernelGGL(kernel, grid, dim3(kThreads), lds, stream, t_time_start, t_time_stop, 0, __VA_ARGS__); \
            t_time_start = t_time_stop = nullptr;                                                                     \
        } else {                                                                                                      \
            hipLaunchKernelGGL(kernel, grid, dim3(kThreads), lds, stream, __VA_ARGS__);                                \
        }                                                                                                             \
    } while (0)

template <int ES_IN, int VEC, int OUT>
static hipError_t launch_t(const CaptureArgs &a, const BatchArgs &b, uint32_t grid, hipStream_t s)
{
    const dim3 g(grid, a.n_batch);
    if (a.summary_mask)
        DMI_LAUNCH_CAPTURE(a.step != nullptr, (capture_kernel<ES_IN, VEC, OUT, true>), g, a.lds_bytes, s,
                           static_cast<const CaptureKernelArgs &>(a), b);
    else
        DMI_LAUNCH_CAPTURE(a.step != nullptr, (capture_kernel<ES_IN, VEC, OUT, false>), g, a.lds_bytes, s,
                           static_cast<const CaptureKernelArgs &>(a), b);
    return hipGetLastError();
}

template <int ES_IN, int VEC>
static hipError_t launch_o(const CaptureArgs &a, const BatchArgs &b, uint32_t grid, hipStream_t s)
{
    const bool raw = a.out_dtype == a.src_dtype;
    if (a.out_dtype == 0) return launch_t<ES_IN, VEC, OUT_NONE>(a, b, grid, s);
    if (raw) return launch_t<ES_IN, VEC, OUT_RAW>(a, b, grid, s);
    if constexpr (ES_IN == 2) {
        if (a.out_dtype == 2) return launch_t<ES_IN, VEC, OUT_FP16>(a, b, grid, s);
        if (a.out_dtype == 4) return launch_t<ES_IN, VEC, OUT_FP8>(a, b, grid, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_capture(const CaptureArgs &a, const BatchArgs &b, uint32_t grid, bool vec16, hipStream_t s)
{
    if (grid == 0 || grid > kMaxGrid || a.n_batch == 0 || a.n_batch > kMaxBatch) return hipErrorInvalidValue;
    const bool four = a.src_dtype == 3;
    if (four) return vec16 ? launch_o<4, 4>(a, b, grid, s) : launch_o<4, 1>(a, b, grid, s);
    return vec16 ? launch_o<2, 8>(a, b, grid, s) : launch_o<2, 1>(a, b, grid, s);
}

template <int OUT>
static hipError_t launch_decode_t(const DecodeArgs &d, const BatchArgs &b, uint32_t n_batch, bool summaries,
                                  hipStream_t s)
{
    const dim3 grid(d.n_wg_rows + 1u, n_batch);
    if (d.keep_mask) {
        if (summaries)
            DMI_LAUNCH_CAPTURE(d.step != nullptr, (capture_decode_kernel<OUT, true, true>), grid, 0, s, d, b);
        else
            DMI_LAUNCH_CAPTURE(d.step != nullptr, (capture_decode_kernel<OUT, false, true>), grid, 0, s, d, b);
    } else {
        if (summaries)
            DMI_LAUNCH_CAPTURE(d.step != nullptr, (capture_decode_kernel<OUT, true, false>), grid, 0, s, d, b);
        else
            DMI_LAUNCH_CAPTURE(d.step != nullptr, (capture_decode_kernel<OUT, false, false>), grid, 0, s, d, b);
    }
    return hipGetLastError();
}

hipError_t launch_capture_decode(const CaptureArgs &a, const BatchArgs &b, hipStream_t s)
{
    if (a.n_src_rows < 0 || a.n_src_rows > 0xFFFFFFFFll) return hipErrorInvalidValue;
    if (a.n_batch == 0 || a.n_batch > kMaxBatch) return hipErrorInvalidValue;
    DecodeArgs d;
    std::memset(&d, 0, sizeof d);
    d.row_stride_b = a.row_stride_b;
    d.rows = a.row_index ? a.row_index : reinterpret_cast<const int32_t *>(a.row_map ? a.row_map : a.row0);
    d.n_wg_rows = a.hdr[9];         // rows listed
    d.ring = a.ring;
    d.cap = a.cap;
    d.ctrl = a.ctrl;
    d.step = a.step;
    d.tail_floor = a.tail_floor;
    d.record_bytes = a.record_bytes;
    d.off_payload = a.off_payload;
    d.off_sum = a.off_sum;
    d.sum_arr = a.sum_arr;
    d.n_src_rows = (uint32_t)a.n_src_rows;
    d.n_reqs = a.n_reqs;
    d.units_per_row = a.units_per_row;
    d.row_first = a.row_first;
    d.flags = (a.drop_newest ? kDecDropNewest : 0u) | (a.rows_consecutive ? kDecConsecutive : 0u) |
              (a.row_index ? kDecIndexed : 0u) | (a.par_in ? kDecParIn : 0u);
    d.node = a.node;
    d.summary_mask = a.summary_mask;
    d.row_elems = a.row_elems;
    d.seq = a.seq;
    d.step_id = a.step_id;
    d.req_table = a.req_table;
    d.cslot = a.cslot;
    d.payload_bytes = a.payload_bytes;
    d.hdr7 = a.hdr[7];
    d.rank_tag = a.rank_tag;
    d.tail_src = a.tail_src;
    d.keep_mask = a.keep_mask;
    if (a.keep_mask && a.n_reqs > 1024u) return hipErrorInvalidValue;
    const bool summ = a.summary_mask != 0;
    if (a.out_dtype == a.src_dtype) return launch_decode_t<OUT_RAW>(d, b, a.n_batch, summ, s);
    switch (a.out_dtype) {
    case 0: return launch_decode_t<OUT_NONE>(d, b, a.n_batch, summ, s);
    case 2: return launch_decode_t<OUT_FP16>(d, b, a.n_batch, summ, s);
    case 4: return launch_decode_t<OUT_FP8>(d, b, a.n_batch, summ, s);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_upload(uint32_t *dst, const uint32_t *words, uint32_t n_words, hipStream_t s)
{
    for (uint32_t o = 0; o < n_words; o += 896u) {
        UploadChunk c;
        const uint32_t n = n_words - o < 896u ? n_words - o : 896u;
        std::memcpy(c.w, words + o, n * 4u);
        hipLaunchKernelGGL(upload_kernel, dim3(1), dim3(kThreads), 0, s, dst + o, c, n);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_ctrl_reset(DevCtrl *ctrl, hipStream_t s)
{
    hipLaunchKernelGGL(ctrl_reset_kernel, dim3(1), dim3(64), 0, s, ctrl);
    return hipGetLastError();
}

hipError_t launch_fetch_slot(const CommitSlot *src, CommitSlot *dst_host, hipStream_t s)
{
    hipLaunchKernelGGL(fetch_slot_kernel, dim3(1), dim3(64), 0, s, src, dst_host);
    return hipGetLastError();
}

hipError_t launch_step_begin(DevCtrl *ctrl, StepParams *step, StepParams v, uint32_t par_from, uint32_t par_to,
                             const uint64_t *host_tail, hipStream_t s)
{
    hipLaunchKernelGGL(step_begin_kernel, dim3(1), dim3(64), 0, s, ctrl, step, v, par_from, par_to, host_tail);
    return hipGetLastError();
}

hipError_t launch_drain_kernel(const uint8_t *ring, uint64_t cap, uint8_t *host_ring, uint64_t host_cap,
                               uint64_t from, uint64_t nbytes, uint32_t grid, hipStream_t s)
{
    hipLaunchKernelGGL(drain_kernel, dim3(grid), dim3(kThreads), 0, s, ring, cap, host_ring, host_cap, from,
                       nbytes);
    return hipGetLastError();
}

}  // namespace dmi
