// HIP kernels of libreft for gfx950 (CDNA4): ragged gather (snapshot pack and in-place XOR parity
// over span tables), ragged scatter (restore) and contiguous k-way XOR (single-loss decode).
//
// All three are HBM-streaming kernels: no arithmetic beyond a 128-bit XOR per 16 bytes and
// source, so the design goal is full-width, coalesced 16-byte accesses with enough of them in
// flight per compute unit.  A workgroup is 256 threads (4 wavefronts of 64).  Work is cut into
// tiles of 2^tile_shift consecutive stream bytes; a launch walks its tiles with a grid-stride loop
// so the grid size (and with it the number of compute units a snapshot occupies next to training
// kernels) is a free parameter.  Consecutive workgroups take consecutive tiles, so the eight XCDs
// (workgroups are dealt to them round-robin) stream through neighbouring addresses together.
//
// Operations (bytes only; see include/reft.h for the paper passages):
//   gather  dst[o] = XOR_s span_s(o)          stream offset o in [lo, hi), spans via pointer tables
//   scatter span(o) = src[o]
//   contig  dst[i] = XOR_s src_s[i]
#include "reft_internal.hpp"

#include <map>
#include <mutex>
#include <tuple>
#include <utility>

namespace reft {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Addresses travel through the kernels as integers (a destination may be a "virtual base" that
// only becomes a valid address once a stream offset is added).  They are turned into pointers in
// the global address space here, so that the accesses compile to global_load / global_store.
#define REFT_GLOBAL __attribute__((address_space(1)))
typedef const REFT_GLOBAL u32x4 *gcptr16;
typedef REFT_GLOBAL u32x4 *gptr16;

__device__ __forceinline__ gcptr16 as_gc16(uint64_t a) { return (gcptr16)a; }
__device__ __forceinline__ gptr16 as_g16(uint64_t a) { return (gptr16)a; }
__device__ __forceinline__ uint8_t ld8(uint64_t a) { return *(const REFT_GLOBAL uint8_t *)a; }
__device__ __forceinline__ void st8(uint64_t a, uint8_t v) { *(REFT_GLOBAL uint8_t *)a = v; }

template <bool NT>
__device__ __forceinline__ u32x4 ld16(gcptr16 p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

template <bool NT>
__device__ __forceinline__ void st16(gptr16 p, u32x4 v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// The 16 bytes that start r bytes (0 < r < 16) into the 32 bytes lo || hi (little endian).
__device__ __forceinline__ u32x4 shift_bytes(u32x4 lo, u32x4 hi, uint32_t r)
{
    const uint32_t q = r >> 2, b = (r & 3u) * 8u;
    uint32_t x0, x1, x2, x3, x4;
    switch (q) {
    case 0:  x0 = lo.x; x1 = lo.y; x2 = lo.z; x3 = lo.w; x4 = hi.x; break;
    case 1:  x0 = lo.y; x1 = lo.z; x2 = lo.w; x3 = hi.x; x4 = hi.y; break;
    case 2:  x0 = lo.z; x1 = lo.w; x2 = hi.x; x3 = hi.y; x4 = hi.z; break;
    default: x0 = lo.w; x1 = hi.x; x2 = hi.y; x3 = hi.z; x4 = hi.w; break;
    }
    if (b) {
        x0 = (x0 >> b) | (x1 << (32u - b));
        x1 = (x1 >> b) | (x2 << (32u - b));
        x2 = (x2 >> b) | (x3 << (32u - b));
        x3 = (x3 >> b) | (x4 << (32u - b));
    }
    u32x4 v = {x0, x1, x2, x3};
    return v;
}

// 16 source bytes at byte address addr + 16*c for any alignment of addr, using only aligned
// 16-byte loads.  Both aligned blocks that are read contain at least one of the wanted bytes, so
// no load reaches outside the 16-byte-aligned hull of the source range.
template <bool NT>
__device__ __forceinline__ u32x4 load_any(uint64_t addr, uint32_t c)
{
    const uint32_t r = (uint32_t)addr & 15u;
    gcptr16 a = as_gc16(addr - r) + c;
    const u32x4 lo = ld16<NT>(a);
    if (r == 0) return lo;
    const u32x4 hi = ld16<NT>(a + 1);
    return shift_bytes(lo, hi, r);
}

// Where the bytes of a piece go: to their global address, or into an LDS image of a destination
// range (image byte 0 stands for the 16-byte aligned address `origin`), from which another wave
// stores them later.
#define REFT_LDS __attribute__((address_space(3)))
struct ToGlobal {
    template <bool NT>
    __device__ __forceinline__ void put16(uint64_t a, u32x4 v) const { st16<NT>(as_g16(a), v); }
    __device__ __forceinline__ void put8(uint64_t a, uint8_t v) const { st8(a, v); }
};
struct ToImage {
    REFT_LDS unsigned char *img;
    uint64_t origin;
    template <bool NT>
    __device__ __forceinline__ void put16(uint64_t a, u32x4 v) const
    {
        *(REFT_LDS u32x4 *)(img + (uint32_t)(a - origin)) = v;
    }
    __device__ __forceinline__ void put8(uint64_t a, uint8_t v) const { img[(uint32_t)(a - origin)] = v; }
};

// The absent second destination of a piece (see xor_piece).
struct NoSink {
    static constexpr bool kActive = false;
    template <bool NT>
    __device__ __forceinline__ void put16(uint64_t, u32x4) const {}
    __device__ __forceinline__ void put8(uint64_t, uint8_t) const {}
};

// One piece: n bytes at destination address d = XOR of the n bytes at each source address s[j].
// The whole workgroup cooperates.  Destination stores are 16-byte aligned: up to 15 head bytes
// and 15 tail bytes are moved bytewise, the body as 16-byte chunks.  If every source is
// co-aligned with the destination (the case for tensors whose sizes and addresses are multiples
// of 16) the body is plain vector loads, U chunks in flight per thread and source; otherwise each
// misaligned source is read as two aligned chunks and byte-shifted in registers.
// With a second sink, the bytes of the first source alone also go to address d2 (+ the same
// offsets) of that sink: the packed copy of one shard beside the parity of all.  d2 must be
// congruent to d modulo 16.
template <int K, int U, bool NT, class Sink = ToGlobal, class Sink2 = NoSink>
__device__ __forceinline__ void xor_piece(uint64_t d, const uint64_t (&s)[K], uint32_t n,
                                          const Sink sink = Sink(), uint64_t d2 = 0,
                                          const Sink2 sink2 = Sink2())
{
    const uint32_t tid = threadIdx.x;
    uint32_t head = (uint32_t)(0 - d) & 15u;
    if (head > n) head = n;
    const uint32_t body = n - head;
    const uint32_t nb = body >> 4;
    const uint32_t tail = body & 15u;

    if (tid < 32) {
        uint32_t i = 0xffffffffu;
        if (tid < head) i = tid;
        else if (tid >= 16 && tid - 16 < tail) i = head + (nb << 4) + (tid - 16);
        if (i != 0xffffffffu) {
            uint8_t v = ld8(s[0] + i);
            sink2.put8(d2 + i, v);
#pragma unroll
            for (int j = 1; j < K; ++j) v ^= ld8(s[j] + i);
            sink.put8(d + i, v);
        }
    }
    if (nb == 0) return;

    const uint64_t da = d + head;
    const uint64_t da2 = d2 + head;
    uint32_t mis = 0;
#pragma unroll
    for (int j = 0; j < K; ++j) mis |= (uint32_t)(s[j] + head) & 15u;

    if (mis == 0) {
        gcptr16 sp[K];
#pragma unroll
        for (int j = 0; j < K; ++j) sp[j] = as_gc16(s[j] + head);
        constexpr uint32_t step = kThreads * U;
        const uint32_t full = nb / step * step;
        for (uint32_t c = tid; c < full; c += step) {
            u32x4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = ld16<NT>(sp[0] + c + u * kThreads);
#pragma unroll
            for (int u = 0; u < U; ++u)
                sink2.template put16<NT>(da2 + ((uint64_t)(c + u * kThreads) << 4), v[u]);
#pragma unroll
            for (int j = 1; j < K; ++j) {
#pragma unroll
                for (int u = 0; u < U; ++u) v[u] ^= ld16<NT>(sp[j] + c + u * kThreads);
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                sink.template put16<NT>(da + ((uint64_t)(c + u * kThreads) << 4), v[u]);
        }
        for (uint32_t c = full + tid; c < nb; c += kThreads) {
            u32x4 v = ld16<NT>(sp[0] + c);
            sink2.template put16<NT>(da2 + ((uint64_t)c << 4), v);
#pragma unroll
            for (int j = 1; j < K; ++j) v ^= ld16<NT>(sp[j] + c);
            sink.template put16<NT>(da + ((uint64_t)c << 4), v);
        }
    } else {
        for (uint32_t c = tid; c < nb; c += kThreads) {
            u32x4 v = load_any<NT>(s[0] + head, c);
            sink2.template put16<NT>(da2 + ((uint64_t)c << 4), v);
#pragma unroll
            for (int j = 1; j < K; ++j) v ^= load_any<NT>(s[j] + head, c);
            sink.template put16<NT>(da + ((uint64_t)c << 4), v);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Tiles that hold many small pieces (many small tensors end to end).
//
// Walking such a tile piece by piece leaves most of the workgroup idle and pays a chain of scalar
// table look-ups per piece.  Instead the slice of the plan that the tile needs - span offsets and
// the span pointers of every source - is staged in LDS once, and the tile is cut into 16-byte
// destination chunks that are dealt to the threads: each thread finds the span that owns its
// chunk by binary search in the LDS copy of the offsets.  A chunk inside one span is moved as a
// vector (realigned in registers if the source is not co-aligned); a chunk that straddles a span
// boundary is assembled byte by byte.  At most kLdsSpans spans are staged per pass; a tile with
// more is handled in several passes.
// ------------------------------------------------------------------------------------------------
constexpr uint32_t kLdsSpans = 256;

// Largest q in [0, n) with off[q] <= x; requires off[0] <= x < off[n].  Zero-length spans
// (off[q] == off[q+1]) are never returned.
__device__ __forceinline__ uint32_t find_span(const uint64_t *off, uint32_t n, uint64_t x)
{
    uint32_t lo = 0, hi = n;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (off[mid] <= x) lo = mid;
        else hi = mid;
    }
    return lo;
}

// XOR over the K sources of the byte at stream offset x, whose span is q or a later one.
template <int K>
__device__ __forceinline__ uint8_t xor_byte_at(const uint64_t *off, const uint64_t (*ptr)[kLdsSpans],
                                               uint32_t &q, uint64_t x)
{
    while (x >= off[q + 1]) ++q;               // x < off[n] bounds the walk
    const uint64_t r = x - off[q];
    uint8_t v = ld8(ptr[0][q] + r);
#pragma unroll
    for (int j = 1; j < K; ++j) v ^= ld8(ptr[j][q] + r);
    return v;
}

// Stream range [o, e) -> dst_vbase + x, spans and pointers of all K sources staged through LDS.
// `i` is a span with off[i] <= o.  If acc, the destination's bytes are the K-th source.
template <int K, bool NT>
__device__ __forceinline__ void gather_small(const PlanTables &pt, const uint64_t *__restrict__ tab,
                                             uint64_t dst_vbase, uint64_t o, uint64_t e, uint32_t i,
                                             uint32_t acc, uint64_t *s_off,
                                             uint64_t (*s_ptr)[kLdsSpans])
{
    const uint32_t tid = threadIdx.x;
    while (o < e) {
        // o < e <= L = off[T] keeps i < T
        const uint32_t n = (uint32_t)(pt.T - i < kLdsSpans ? pt.T - i : kLdsSpans);
        __syncthreads();                                   // the previous pass is done with LDS
        for (uint32_t q = tid; q <= n; q += kThreads) s_off[q] = pt.off[i + q];
#pragma unroll
        for (int j = 0; j < K; ++j) {
            if (acc && j == K - 1) {
                // the destination as a source: "span pointer" = address of the span's first byte
                for (uint32_t q = tid; q < n; q += kThreads) s_ptr[j][q] = dst_vbase + pt.off[i + q];
            } else {
                for (uint32_t q = tid; q < n; q += kThreads)
                    s_ptr[j][q] = tab[(uint64_t)j * pt.T + i + q];
            }
        }
        __syncthreads();
        const uint64_t sub_e = s_off[n] < e ? s_off[n] : e;
        if (sub_e > o) {
            const uint64_t d0 = dst_vbase + o;
            uint32_t len = (uint32_t)(sub_e - o);
            uint32_t head = (uint32_t)(0 - d0) & 15u;
            if (head > len) head = len;
            const uint32_t nb = (len - head) >> 4;
            const uint32_t tail = (len - head) & 15u;
            if (tid < 32) {                                // edge bytes, one per thread
                uint32_t b = 0xffffffffu;
                if (tid < head) b = tid;
                else if (tid >= 16 && tid - 16 < tail) b = head + (nb << 4) + (tid - 16);
                if (b != 0xffffffffu) {
                    uint32_t q = find_span(s_off, n, o + b);
                    st8(d0 + b, xor_byte_at<K>(s_off, s_ptr, q, o + b));
                }
            }
            const uint64_t x0 = o + head;
            gptr16 dp = as_g16(d0 + head);
            for (uint32_t c = tid; c < nb; c += kThreads) {
                const uint64_t x = x0 + ((uint64_t)c << 4);
                uint32_t q = find_span(s_off, n, x);
                u32x4 v;
                if (x + 16 <= s_off[q + 1]) {              // the chunk lies inside one span
                    const uint64_t r = x - s_off[q];
                    v = load_any<NT>(s_ptr[0][q] + r, 0);
#pragma unroll
                    for (int j = 1; j < K; ++j) v ^= load_any<NT>(s_ptr[j][q] + r, 0);
                } else {                                   // it straddles a span boundary
                    uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
                    for (int b = 0; b < 16; ++b)
                        w[b >> 2] |= (uint32_t)xor_byte_at<K>(s_off, s_ptr, q, x + b) << ((b & 3) * 8);
                    v.x = w[0]; v.y = w[1]; v.z = w[2]; v.w = w[3];
                }
                st16<NT>(dp + c, v);
            }
        }
        o = sub_e > o ? sub_e : o;
        i += n;
    }
}

// Stream range [o, e) at src_vbase + x -> the spans' own places, span table staged through LDS.
template <bool NT>
__device__ __forceinline__ void scatter_small(const PlanTables &pt, const uint64_t *__restrict__ tab,
                                              uint64_t src_vbase, uint64_t o, uint64_t e, uint32_t i,
                                              uint64_t *s_off, uint64_t (*s_ptr)[kLdsSpans])
{
    const uint32_t tid = threadIdx.x;
    while (o < e) {
        const uint32_t n = (uint32_t)(pt.T - i < kLdsSpans ? pt.T - i : kLdsSpans);
        __syncthreads();
        for (uint32_t q = tid; q <= n; q += kThreads) s_off[q] = pt.off[i + q];
        for (uint32_t q = tid; q < n; q += kThreads) s_ptr[0][q] = tab[i + q];
        __syncthreads();
        const uint64_t sub_e = s_off[n] < e ? s_off[n] : e;
        // Are all destinations of this pass co-aligned with the source stream?  (True for tensors
        // whose sizes and addresses are multiples of 16.)  If not, 16-byte source chunks would
        // have to be stored in narrow pieces; the piece routine, which realigns on the load side,
        // is the better tool then, fed from the LDS copy of the tables.
        int mis = 0;
        for (uint32_t q = tid; q < n; q += kThreads)
            if (s_off[q + 1] > s_off[q] && ((s_ptr[0][q] - (src_vbase + s_off[q])) & 15u)) mis = 1;
        mis = __syncthreads_or(mis);
        if (sub_e > o && mis) {
            uint64_t x = o;
            uint32_t q = find_span(s_off, n, x);
            while (x < sub_e) {
                while (s_off[q + 1] <= x) ++q;                 // x < sub_e <= off[n]
                uint64_t pe = s_off[q + 1] < sub_e ? s_off[q + 1] : sub_e;
                const uint64_t src1[1] = {src_vbase + x};
                xor_piece<1, 1, NT>(s_ptr[0][q] + (x - s_off[q]), src1, (uint32_t)(pe - x));
                x = pe;
            }
        } else if (sub_e > o) {
            // chunks are aligned on the (contiguous) source side; each goes to its span's place
            const uint64_t s0 = src_vbase + o;
            uint32_t len = (uint32_t)(sub_e - o);
            uint32_t head = (uint32_t)(0 - s0) & 15u;
            if (head > len) head = len;
            const uint32_t nb = (len - head) >> 4;
            const uint32_t tail = (len - head) & 15u;
            if (tid < 32) {
                uint32_t b = 0xffffffffu;
                if (tid < head) b = tid;
                else if (tid >= 16 && tid - 16 < tail) b = head + (nb << 4) + (tid - 16);
                if (b != 0xffffffffu) {
                    const uint64_t x = o + b;
                    const uint32_t q = find_span(s_off, n, x);
                    st8(s_ptr[0][q] + (x - s_off[q]), ld8(s0 + b));
                }
            }
            const uint64_t x0 = o + head;
            gcptr16 sp = as_gc16(s0 + head);
            for (uint32_t c = tid; c < nb; c += kThreads) {
                const uint64_t x = x0 + ((uint64_t)c << 4);
                uint32_t q = find_span(s_off, n, x);
                const u32x4 v = ld16<NT>(sp + c);
                const uint64_t d = s_ptr[0][q] + (x - s_off[q]);
                if (x + 16 <= s_off[q + 1] && (d & 15u) == 0) {
                    st16<NT>(as_g16(d), v);
                } else {                                   // a span boundary inside the chunk
                    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int b = 0; b < 16; ++b) {
                        const uint64_t xb = x + b;
                        while (xb >= s_off[q + 1]) ++q;    // xb < sub_e <= off[n] bounds the walk
                        st8(s_ptr[0][q] + (xb - s_off[q]), (uint8_t)(w[b >> 2] >> ((b & 3) * 8)));
                    }
                }
            }
        }
        o = sub_e > o ? sub_e : o;
        i += n;
    }
}

// destination of stream byte o  <-  XOR over rows j < K of (tab[j*T + span(o)] + offset of o in
// its span).  The destination is dst_vbase + o, or, if dtab is not null, ragged as well:
// dtab[span(o)] + offset.  With acc != 0 only K-1 rows are read and the destination itself is the
// K-th source.
template <int K, int U, bool NT>
__global__ void __launch_bounds__(kThreads)
k_gather(PlanTables pt, const uint64_t *__restrict__ tab, const uint64_t *__restrict__ dtab,
         uint64_t dst_vbase, uint64_t lo, uint64_t hi, uint32_t acc, uint32_t small_pieces)
{
    __shared__ uint64_t s_off[kLdsSpans + 1];
    __shared__ uint64_t s_ptr[K][kLdsSpans];
    const uint32_t sh = pt.tile_shift;
    const uint64_t t_last = (hi - 1) >> sh;
    const uint64_t t_end = (pt.L - 1) >> sh;              // last tile of the stream
    for (uint64_t t = (lo >> sh) + blockIdx.x; t <= t_last; t += gridDim.x) {
        uint64_t o = t << sh;
        uint64_t e = o + (1ull << sh);
        if (o < lo) o = lo;
        if (e > hi) e = hi;
        uint32_t i = pt.first_span[t];
        // spans that start inside this tile (an upper bound of its pieces minus one)
        const uint32_t i_next = t < t_end ? pt.first_span[t + 1] : (uint32_t)(pt.T - 1);
        if (dtab == nullptr && i_next - i >= small_pieces) {
            gather_small<K, NT>(pt, tab, dst_vbase, o, e, i, acc, s_off, s_ptr);
            continue;
        }
        while (o < e) {
            // o < e <= L = off[T], so a span with off[i+1] > o exists at or after i
            while (pt.off[i + 1] <= o) ++i;
            const uint64_t so = pt.off[i];
            uint64_t pe = pt.off[i + 1];
            if (pe > e) pe = e;
            const uint64_t d = dtab ? dtab[i] + (o - so) : dst_vbase + o;
            uint64_t s[K];
#pragma unroll
            for (int j = 0; j < K - 1; ++j) s[j] = tab[(uint64_t)j * pt.T + i] + (o - so);
            // accumulate mode: the destination's current bytes are the last source (each byte
            // is read and then written by the same thread, so in-place is safe)
            s[K - 1] = acc ? d : tab[(uint64_t)(K - 1) * pt.T + i] + (o - so);
            xor_piece<K, U, NT>(d, s, (uint32_t)(pe - o));
            o = pe;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Gather with write bursts (many sources, one pass).
//
// Measured on this part: a stream of reads runs at about 7 TB/s, but as soon as writes are mixed
// into it, even a few, the whole stream drops to 5.2 - 5.9 TB/s; the same bytes written in short
// chip-wide bursts cost far less.  So this variant separates the two in time.  A workgroup has
// four reader waves and one writer wave.  The readers XOR one stage (stage_bytes of the stream)
// after another into the two halves of an LDS double buffer and never touch the destination.
// The writer wave stores stage r-1 from its half while the readers fill the other half with stage
// r - but not before every workgroup of the grid has finished reading its stage r-1, so that
// all writer waves of the chip fire together.  That meeting is only a matter of timing: it is a
// counter the writer wave polls at most max_polls times per round (readers never wait for another
// workgroup), a writer that polls in vain stops waiting for the next 1, 2, 4, ... 64 rounds (so a
// slow workgroup, or one that is not resident, costs the others next to nothing), and the result
// does not depend on it.  The grid is persistent (the launch wrappers size it so that all
// workgroups are resident); workgroup b takes stages b, b + grid, ...
//
// The LDS image of a stage is laid out like the destination: the byte of stream offset o sits
// where address vb + o would fall relative to a 16-byte boundary.  For a contiguous destination
// vb is its virtual base.  For a ragged one (dtab), every span's place must have the same
// alignment relative to its stream offset, (dtab[i] - off[i]) mod 16 = vb mod 16 for all spans
// with bytes (the host checks this); then aligned 16-byte chunks of the image are aligned
// 16-byte chunks of every destination span.
//
// ctr: 9 counters kCtrStride words apart, all zero at launch.  Workgroups arrive on counter
// (blockIdx.x & 7); every arrival that completes a multiple of the group's size bumps counter 8,
// the only one polled, so counter 8 tells how many rounds the groups have completed between them.
// ------------------------------------------------------------------------------------------------
constexpr int kBurstThreads = kThreads + 64;
constexpr uint32_t kCtrStride = 64;

// One wave moves len bytes from an LDS image to global address d (img is the byte for d; img and d
// have the same alignment mod 16).
template <bool NT>
__device__ __forceinline__ void emit_piece(uint64_t d, REFT_LDS const unsigned char *img,
                                           uint32_t len, uint32_t lane)
{
    uint32_t head = (uint32_t)(0 - d) & 15u;
    if (head > len) head = len;
    const uint32_t nb = (len - head) >> 4;
    const uint32_t tail = (len - head) & 15u;
    if (lane < head) {
        st8(d + lane, img[lane]);
    } else if (lane >= 16 && lane - 16 < tail) {
        const uint32_t b = head + (nb << 4) + (lane - 16);
        st8(d + b, img[b]);
    }
    if (nb) {
        gptr16 dp = as_g16(d + head);
        REFT_LDS const u32x4 *ip = (REFT_LDS const u32x4 *)(img + head);
#pragma unroll 8
        for (uint32_t c = lane; c < nb; c += 64) st16<NT>(dp + c, ip[c]);
    }
}

// The rounds of a burst kernel.  read(st, img) is run by the 256 reader threads and puts stage st
// into the LDS image at img; emit(st, img, lane) is run by the writer wave and stores the image.
// With NIMG = 2 every half holds a second image behind the two of the first (at + 2 * (stage + 16)).
template <int NIMG = 1, class Read, class Emit>
__device__ __forceinline__ void burst_rounds(uint64_t nstages, uint32_t stage, uint32_t *ctr,
                                             uint32_t max_polls, uint32_t nap, Read read, Emit emit)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char burst_lds[];
    REFT_LDS unsigned char *lds = (REFT_LDS unsigned char *)burst_lds;
    const uint32_t half = stage + 16;                  // an image may start up to 15 bytes in
    const uint32_t lane = threadIdx.x & 63;
    const bool writer = threadIdx.x >= kThreads;
    const uint32_t G = gridDim.x, g = blockIdx.x & 7;
    const uint64_t rounds = (nstages + G - 1) / G;
    const uint32_t members = (G - g + 7) >> 3;         // workgroups that arrive on counter g
    const uint32_t ngroups = G < 8 ? G : 8;
    uint32_t skip = 0, backoff = 0;                    // writer wave: rounds left without waiting
    // writer wave, lane 0: how its rounds went (met, timed out, not waited), kept in LDS behind
    // the two images so that the bookkeeping costs the kernels no registers
    REFT_LDS uint32_t *tally = (REFT_LDS uint32_t *)(lds + 2 * NIMG * half);
    if (threadIdx.x == kThreads) tally[0] = tally[1] = tally[2] = 0;

    for (uint64_t r = 0; r <= rounds; ++r) {
        if (!writer) {
            const uint64_t st = r * G + blockIdx.x;
            if (r < rounds && st < nstages) read(st, lds + (uint32_t)(r & 1) * half);
        } else if (r > 0) {
            if (skip) {
                --skip;
                if (lane == 0) tally[2] += 1;
            } else if (max_polls) {
                const uint32_t want = ngroups * (uint32_t)r;   // every group done with round r-1
                for (uint32_t n = 0;;) {
                    uint32_t v = 0;
                    if (lane == 0)
                        v = __hip_atomic_load(ctr + 8 * kCtrStride, __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT);
                    v = __builtin_amdgcn_readfirstlane(v);
                    if (v >= want) {
                        backoff = 0;
                        if (lane == 0) tally[0] += 1;
                        break;
                    }
                    if (++n >= max_polls) {
                        // a straggler: write without the others for 1, 2, 4, ... 64 rounds
                        backoff = backoff == 0 ? 1 : backoff < 64 ? backoff * 2 : 64;
                        skip = backoff;
                        if (lane == 0) tally[1] += 1;
                        break;
                    }
                    for (uint32_t z = 0; z < nap; ++z) __builtin_amdgcn_s_sleep(16);
                }
            }
            const uint64_t st = (r - 1) * G + blockIdx.x;
            if (st < nstages) emit(st, lds + (uint32_t)((r - 1) & 1) * half, lane);
        }
        __syncthreads();       // stage r is complete in LDS; stage r-1 has left its half
        if (writer && lane == 0 && r < rounds && max_polls) {
            const uint32_t old = __hip_atomic_fetch_add(ctr + g * kCtrStride, 1u, __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_AGENT);
            if ((old + 1) % members == 0)     // whichever round the arriving workgroup is in
                __hip_atomic_fetch_add(ctr + 8 * kCtrStride, 1u, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    // diagnostics (three adds per workgroup and launch): rounds in which the writer wave saw the
    // meeting complete, ran out of polls, or did not wait at all
    if (writer && lane == 0 && max_polls) {
        uint32_t *diag = ctr + kBurstDiagWord;
        __hip_atomic_fetch_add(diag + 0, tally[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_add(diag + 1, tally[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_add(diag + 2, tally[2], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <int K, int U, bool NT>
__global__ void __launch_bounds__(kBurstThreads)
k_gather_burst(PlanTables pt, const uint64_t *__restrict__ tab, const uint64_t *__restrict__ dtab,
               uint64_t vb, uint64_t lo, uint64_t hi, uint32_t acc, uint32_t stage, uint32_t *ctr,
               uint32_t max_polls, uint32_t nap)
{
    const uint64_t nstages = (hi - lo + stage - 1) / stage;
    burst_rounds(
        nstages, stage, ctr, max_polls, nap,
        [&](uint64_t st, REFT_LDS unsigned char *img) {
            uint64_t o = lo + st * stage;
            uint64_t e = o + stage;
            if (e > hi) e = hi;
            const ToImage sink{img, (vb + o) & ~15ull};
            uint32_t i = pt.first_span[o >> pt.tile_shift];
            while (o < e) {
                // o < e <= L = off[T], so a span with off[i+1] > o exists at or after i
                while (pt.off[i + 1] <= o) ++i;
                const uint64_t so = pt.off[i];
                uint64_t pe = pt.off[i + 1];
                if (pe > e) pe = e;
                uint64_t s[K];
#pragma unroll
                for (int j = 0; j < K - 1; ++j) s[j] = tab[(uint64_t)j * pt.T + i] + (o - so);
                // accumulate mode: the destination's current bytes are the last source (a stage
                // of the destination is read and, a round later, written by this workgroup only)
                s[K - 1] = !acc ? tab[(uint64_t)(K - 1) * pt.T + i] + (o - so)
                                : dtab ? dtab[i] + (o - so) : vb + o;
                xor_piece<K, U, NT, ToImage>(vb + o, s, (uint32_t)(pe - o), sink);
                o = pe;
            }
        },
        [&](uint64_t st, REFT_LDS const unsigned char *img, uint32_t lane) {
            uint64_t o = lo + st * stage;
            const uint64_t e = o + stage < hi ? o + stage : hi;
            // image byte of stream offset x: img0[x - o]
            REFT_LDS const unsigned char *img0 = img + ((uint32_t)(vb + o) & 15u);
            if (dtab == nullptr) {
                emit_piece<NT>(vb + o, img0, (uint32_t)(e - o), lane);
            } else {
                const uint64_t o0 = o;
                uint32_t i = pt.first_span[o >> pt.tile_shift];
                while (o < e) {
                    while (pt.off[i + 1] <= o) ++i;
                    const uint64_t so = pt.off[i];
                    const uint64_t pe = pt.off[i + 1] < e ? pt.off[i + 1] : e;
                    emit_piece<NT>(dtab[i] + (o - so), img0 + (uint32_t)(o - o0), (uint32_t)(pe - o),
                                   lane);
                    o = pe;
                }
            }
        });
}

// The parity of K rows into a contiguous destination and, in the same pass, the packed stream of
// row 0 into a second contiguous destination (fused pack + encode: the first row is read once
// for both).  vb2 is the virtual base of the packed copy, congruent to vb modulo 16.  Two LDS
// images per half, so a workgroup needs 4 * (stage + 16) bytes of LDS.
template <int K, int U, bool NT>
__global__ void __launch_bounds__(kBurstThreads)
k_gather_burst_pack(PlanTables pt, const uint64_t *__restrict__ tab, uint64_t vb, uint64_t vb2,
                    uint64_t lo, uint64_t hi, uint32_t stage, uint32_t *ctr, uint32_t max_polls,
                    uint32_t nap)
{
    const uint64_t nstages = (hi - lo + stage - 1) / stage;
    const uint32_t second = 2 * (stage + 16);          // the second image of a half
    burst_rounds<2>(
        nstages, stage, ctr, max_polls, nap,
        [&](uint64_t st, REFT_LDS unsigned char *img) {
            uint64_t o = lo + st * stage;
            uint64_t e = o + stage;
            if (e > hi) e = hi;
            const ToImage sink{img, (vb + o) & ~15ull};
            const ToImage sink2{img + second, (vb2 + o) & ~15ull};
            uint32_t i = pt.first_span[o >> pt.tile_shift];
            while (o < e) {
                while (pt.off[i + 1] <= o) ++i;        // o < e <= L = off[T]
                const uint64_t so = pt.off[i];
                uint64_t pe = pt.off[i + 1];
                if (pe > e) pe = e;
                uint64_t s[K];
#pragma unroll
                for (int j = 0; j < K; ++j) s[j] = tab[(uint64_t)j * pt.T + i] + (o - so);
                xor_piece<K, U, NT, ToImage, ToImage>(vb + o, s, (uint32_t)(pe - o), sink, vb2 + o,
                                                      sink2);
                o = pe;
            }
        },
        [&](uint64_t st, REFT_LDS const unsigned char *img, uint32_t lane) {
            const uint64_t o = lo + st * stage;
            const uint64_t e = o + stage < hi ? o + stage : hi;
            emit_piece<NT>(vb + o, img + ((uint32_t)(vb + o) & 15u), (uint32_t)(e - o), lane);
            emit_piece<NT>(vb2 + o, img + second + ((uint32_t)(vb2 + o) & 15u), (uint32_t)(e - o), lane);
        });
}

// dst[i] = XOR_j src.p[j][i], i in [0, L), with write bursts
template <int K, int U, bool NT>
__global__ void __launch_bounds__(kBurstThreads)
k_xor_contig_burst(SrcBases src, uint64_t dst, uint64_t L, uint32_t stage, uint32_t *ctr,
                   uint32_t max_polls, uint32_t nap)
{
    const uint64_t nstages = (L + stage - 1) / stage;
    burst_rounds(
        nstages, stage, ctr, max_polls, nap,
        [&](uint64_t st, REFT_LDS unsigned char *img) {
            const uint64_t o = st * stage;
            const uint64_t n = L - o < stage ? L - o : stage;
            uint64_t s[K];
#pragma unroll
            for (int j = 0; j < K; ++j) s[j] = src.p[j] + o;
            xor_piece<K, U, NT, ToImage>(dst + o, s, (uint32_t)n, ToImage{img, (dst + o) & ~15ull});
        },
        [&](uint64_t st, REFT_LDS const unsigned char *img, uint32_t lane) {
            const uint64_t o = st * stage;
            const uint64_t n = L - o < stage ? L - o : stage;
            emit_piece<NT>(dst + o, img + ((uint32_t)(dst + o) & 15u), (uint32_t)n, lane);
        });
}

__global__ void k_zero_words(uint32_t *p, uint32_t n)
{
    for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0;
}

// tab[span(o)] + offset of o in its span  <-  src_vbase + o
template <int U, bool NT>
__global__ void __launch_bounds__(kThreads)
k_scatter(PlanTables pt, const uint64_t *__restrict__ tab, uint64_t src_vbase, uint64_t lo,
          uint64_t hi, uint32_t small_pieces)
{
    __shared__ uint64_t s_off[kLdsSpans + 1];
    __shared__ uint64_t s_ptr[1][kLdsSpans];
    const uint32_t sh = pt.tile_shift;
    const uint64_t t_last = (hi - 1) >> sh;
    const uint64_t t_end = (pt.L - 1) >> sh;
    for (uint64_t t = (lo >> sh) + blockIdx.x; t <= t_last; t += gridDim.x) {
        uint64_t o = t << sh;
        uint64_t e = o + (1ull << sh);
        if (o < lo) o = lo;
        if (e > hi) e = hi;
        uint32_t i = pt.first_span[t];
        const uint32_t i_next = t < t_end ? pt.first_span[t + 1] : (uint32_t)(pt.T - 1);
        if (i_next - i >= small_pieces) {
            scatter_small<NT>(pt, tab, src_vbase, o, e, i, s_off, s_ptr);
            continue;
        }
        while (o < e) {
            while (pt.off[i + 1] <= o) ++i;
            const uint64_t so = pt.off[i];
            uint64_t pe = pt.off[i + 1];
            if (pe > e) pe = e;
            const uint64_t s[1] = {src_vbase + o};
            xor_piece<1, U, NT>(tab[i] + (o - so), s, (uint32_t)(pe - o));
            o = pe;
        }
    }
}

// dst[i] = XOR_j src.p[j][i], i in [0, L)
template <int K, int U, bool NT>
__global__ void __launch_bounds__(kThreads)
k_xor_contig(SrcBases src, uint64_t dst, uint64_t L, uint32_t sh)
{
    const uint64_t ntiles = (L + (1ull << sh) - 1) >> sh;
    for (uint64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const uint64_t o = t << sh;
        uint64_t n = L - o;
        if (n > (1ull << sh)) n = 1ull << sh;
        uint64_t s[K];
#pragma unroll
        for (int j = 0; j < K; ++j) s[j] = src.p[j] + o;
        xor_piece<K, U, NT>(dst + o, s, (uint32_t)n);
    }
}

// ------------------------------------------------------------------------------------------------
// launch wrappers: pick the instantiation for (number of sources, unroll, non-temporal)
// ------------------------------------------------------------------------------------------------
static uint32_t grid_for(uint64_t ntiles, const LaunchCfg &cfg)
{
    uint64_t g = ntiles < cfg.max_wgs ? ntiles : cfg.max_wgs;
    return (uint32_t)(g < 1 ? 1 : g);
}

#define REFT_PICK_UNT(KERNEL, K)                                                                  \
    (cfg.nontemporal                                                                              \
         ? (cfg.unroll == 1 ? KERNEL<K, 1, true> : cfg.unroll == 2 ? KERNEL<K, 2, true>           \
                                                                   : KERNEL<K, 4, true>)          \
         : (cfg.unroll == 1 ? KERNEL<K, 1, false> : cfg.unroll == 2 ? KERNEL<K, 2, false>         \
                                                                    : KERNEL<K, 4, false>))

#define REFT_PICK_K(KERNEL, fn, nsrc)                                                             \
    switch (nsrc) {                                                                               \
    case 1: fn = REFT_PICK_UNT(KERNEL, 1); break;                                                 \
    case 2: fn = REFT_PICK_UNT(KERNEL, 2); break;                                                 \
    case 3: fn = REFT_PICK_UNT(KERNEL, 3); break;                                                 \
    case 4: fn = REFT_PICK_UNT(KERNEL, 4); break;                                                 \
    case 5: fn = REFT_PICK_UNT(KERNEL, 5); break;                                                 \
    case 6: fn = REFT_PICK_UNT(KERNEL, 6); break;                                                 \
    case 7: fn = REFT_PICK_UNT(KERNEL, 7); break;                                                 \
    case 8: fn = REFT_PICK_UNT(KERNEL, 8); break;                                                 \
    default: return hipErrorInvalidValue;                                                         \
    }

hipError_t launch_gather(const PlanTables &pt, const uint64_t *tab, int nrows, bool acc,
                         const uint64_t *dtab, uint64_t dst_vbase, uint64_t lo, uint64_t hi,
                         const LaunchCfg &cfg, hipStream_t stream)
{
    if (lo >= hi) return hipSuccess;
    if (hi > pt.L) return hipErrorInvalidValue;
    void (*fn)(PlanTables, const uint64_t *, const uint64_t *, uint64_t, uint64_t, uint64_t,
               uint32_t, uint32_t) = nullptr;
    const int nsrc = nrows + (acc ? 1 : 0);
    REFT_PICK_K(k_gather, fn, nsrc)
    const uint64_t ntiles = ((hi - 1) >> pt.tile_shift) - (lo >> pt.tile_shift) + 1;
    hipLaunchKernelGGL(fn, dim3(grid_for(ntiles, cfg)), dim3(kThreads), 0, stream, pt, tab, dtab,
                       dst_vbase, lo, hi, acc ? 1u : 0u, cfg.small_pieces);
    return hipGetLastError();
}

// Workgroups of the burst kernel that fit on one compute unit with `lds` bytes of LDS each
// (looked up once per instantiation; the first call also lifts the kernel's LDS limit).
static hipError_t burst_occupancy(const void *fn, size_t lds, int *per_cu)
{
    static std::mutex mu;
    static std::map<std::tuple<int, const void *, size_t>, int> known;   // per device
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    auto it = known.find(std::make_tuple(dev, fn, lds));
    if (it == known.end()) {
        e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        int n = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, fn, kBurstThreads, lds);
        if (e != hipSuccess) return e;
        it = known.emplace(std::make_tuple(dev, fn, lds), n).first;
    }
    *per_cu = it->second;
    return hipSuccess;
}

static bool burst_cfg_ok(const BurstCfg &bc)
{
    return bc.ctr && bc.stage_bytes >= 4096 && bc.stage_bytes % 4096 == 0 &&
           bc.stage_bytes <= 65536 && bc.wgs_per_cu >= 1 && bc.num_cus >= 1;
}

// Grid of a burst launch: every workgroup resident at once.
static hipError_t burst_grid(const void *fn, uint64_t nstages, const LaunchCfg &cfg,
                             const BurstCfg &bc, size_t *lds, uint32_t *grid, int images = 1)
{
    // one image per half (two with the fused pack) and the writer's tally
    *lds = 2 * (size_t)images * ((size_t)bc.stage_bytes + 16) + 16;
    int per_cu = 0;
    hipError_t e = burst_occupancy(fn, *lds, &per_cu);
    if (e != hipSuccess) return e;
    if (per_cu < 1) return hipErrorInvalidValue;
    if ((uint32_t)per_cu > bc.wgs_per_cu) per_cu = (int)bc.wgs_per_cu;
    uint64_t g = (uint64_t)per_cu * bc.num_cus;
    if (g > cfg.max_wgs) g = cfg.max_wgs;
    if (g > nstages) g = nstages;
    *grid = (uint32_t)g;
    return hipSuccess;
}

hipError_t launch_gather_burst(const PlanTables &pt, const uint64_t *tab, int nrows, bool acc,
                               const uint64_t *dtab, uint64_t vb, uint64_t lo, uint64_t hi,
                               const LaunchCfg &cfg, const BurstCfg &bc, hipStream_t stream)
{
    if (lo >= hi) return hipSuccess;
    if (hi > pt.L || !burst_cfg_ok(bc)) return hipErrorInvalidValue;
    void (*fn)(PlanTables, const uint64_t *, const uint64_t *, uint64_t, uint64_t, uint64_t, uint32_t,
               uint32_t, uint32_t *, uint32_t, uint32_t) = nullptr;
    const int nsrc = nrows + (acc ? 1 : 0);
    REFT_PICK_K(k_gather_burst, fn, nsrc)
    size_t lds = 0;
    uint32_t grid = 0;
    const uint64_t nstages = (hi - lo + bc.stage_bytes - 1) / bc.stage_bytes;
    hipError_t e = burst_grid((const void *)fn, nstages, cfg, bc, &lds, &grid);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(256), 0, stream, bc.ctr, 9 * kCtrStride);
    hipLaunchKernelGGL(fn, dim3(grid), dim3(kBurstThreads), lds, stream, pt, tab, dtab, vb, lo, hi,
                       acc ? 1u : 0u, bc.stage_bytes, bc.ctr, bc.max_polls, bc.nap);
    return hipGetLastError();
}

hipError_t launch_gather_burst_pack(const PlanTables &pt, const uint64_t *tab, int nrows, uint64_t vb,
                                    uint64_t vb2, uint64_t lo, uint64_t hi, const LaunchCfg &cfg,
                                    const BurstCfg &bc, hipStream_t stream)
{
    if (lo >= hi) return hipSuccess;
    if (hi > pt.L || !burst_cfg_ok(bc) || ((vb ^ vb2) & 15u)) return hipErrorInvalidValue;
    if (4 * ((size_t)bc.stage_bytes + 16) + 16 > 160 * 1024) return hipErrorInvalidValue;
    void (*fn)(PlanTables, const uint64_t *, uint64_t, uint64_t, uint64_t, uint64_t, uint32_t,
               uint32_t *, uint32_t, uint32_t) = nullptr;
    switch (nrows) {                                   // one instantiation per row count
    case 1: fn = k_gather_burst_pack<1, 4, true>; break;
    case 2: fn = k_gather_burst_pack<2, 4, true>; break;
    case 3: fn = k_gather_burst_pack<3, 4, true>; break;
    case 4: fn = k_gather_burst_pack<4, 4, true>; break;
    case 5: fn = k_gather_burst_pack<5, 4, true>; break;
    case 6: fn = k_gather_burst_pack<6, 4, true>; break;
    case 7: fn = k_gather_burst_pack<7, 4, true>; break;
    case 8: fn = k_gather_burst_pack<8, 4, true>; break;
    default: return hipErrorInvalidValue;
    }
    size_t lds = 0;
    uint32_t grid = 0;
    const uint64_t nstages = (hi - lo + bc.stage_bytes - 1) / bc.stage_bytes;
    hipError_t e = burst_grid((const void *)fn, nstages, cfg, bc, &lds, &grid, 2);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(256), 0, stream, bc.ctr, 9 * kCtrStride);
    hipLaunchKernelGGL(fn, dim3(grid), dim3(kBurstThreads), lds, stream, pt, tab, vb, vb2, lo, hi,
                       bc.stage_bytes, bc.ctr, bc.max_polls, bc.nap);
    return hipGetLastError();
}

hipError_t launch_xor_contig_burst(const SrcBases &src, int nsrc, uint64_t dst, uint64_t L,
                                   const LaunchCfg &cfg, const BurstCfg &bc, hipStream_t stream)
{
    if (L == 0) return hipSuccess;
    if (!burst_cfg_ok(bc)) return hipErrorInvalidValue;
    void (*fn)(SrcBases, uint64_t, uint64_t, uint32_t, uint32_t *, uint32_t, uint32_t) = nullptr;
    REFT_PICK_K(k_xor_contig_burst, fn, nsrc)
    size_t lds = 0;
    uint32_t grid = 0;
    const uint64_t nstages = (L + bc.stage_bytes - 1) / bc.stage_bytes;
    hipError_t e = burst_grid((const void *)fn, nstages, cfg, bc, &lds, &grid);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(256), 0, stream, bc.ctr, 9 * kCtrStride);
    hipLaunchKernelGGL(fn, dim3(grid), dim3(kBurstThreads), lds, stream, src, dst, L,
                       bc.stage_bytes, bc.ctr, bc.max_polls, bc.nap);
    return hipGetLastError();
}

hipError_t launch_scatter(const PlanTables &pt, const uint64_t *tab, uint64_t src_vbase,
                          uint64_t lo, uint64_t hi, const LaunchCfg &cfg, hipStream_t stream)
{
    if (lo >= hi) return hipSuccess;
    if (hi > pt.L) return hipErrorInvalidValue;
    void (*fn)(PlanTables, const uint64_t *, uint64_t, uint64_t, uint64_t, uint32_t) =
        cfg.nontemporal
            ? (cfg.unroll == 1 ? k_scatter<1, true> : cfg.unroll == 2 ? k_scatter<2, true>
                                                                      : k_scatter<4, true>)
            : (cfg.unroll == 1 ? k_scatter<1, false> : cfg.unroll == 2 ? k_scatter<2, false>
                                                                       : k_scatter<4, false>);
    const uint64_t ntiles = ((hi - 1) >> pt.tile_shift) - (lo >> pt.tile_shift) + 1;
    hipLaunchKernelGGL(fn, dim3(grid_for(ntiles, cfg)), dim3(kThreads), 0, stream, pt, tab,
                       src_vbase, lo, hi, cfg.small_pieces);
    return hipGetLastError();
}

hipError_t launch_xor_contig(const SrcBases &src, int nsrc, uint64_t dst, uint64_t L,
                             uint32_t tile_shift, const LaunchCfg &cfg, hipStream_t stream)
{
    if (L == 0) return hipSuccess;
    void (*fn)(SrcBases, uint64_t, uint64_t, uint32_t) = nullptr;
    REFT_PICK_K(k_xor_contig, fn, nsrc)
    const uint64_t ntiles = (L + (1ull << tile_shift) - 1) >> tile_shift;
    hipLaunchKernelGGL(fn, dim3(grid_for(ntiles, cfg)), dim3(kThreads), 0, stream, src, dst, L,
                       tile_shift);
    return hipGetLastError();
}

}  // namespace reft
