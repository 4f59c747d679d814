/*
 * CPU oracle for the in-memory checkpointing hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, obviously-correct statement of what the GPU library must produce.  It is
 * linked by nothing in the product: only the tests, the smoke check and the bench's CPU-baseline
 * leg may load it.  It shares no code, header, table or helper with the HIP path.
 *
 * What it states (all on raw bytes; floating-point values are never interpreted):
 *
 *   stream   A rank's snapshot is its state tensors laid end to end as one flat vector, in the
 *            caller's order, with no header and no padding (the flat "vectorized W" that
 *            SplitParameter of Algorithm 1 cuts by index; section 1 says what a snapshot holds,
 *            section 7.1 that it is lossless).
 *   bucket   A bucket is a consecutive byte range of that flat vector; bucket b is stored at host
 *            offset B_b, so the host copy equals the stream whatever the bucket lengths are
 *            (generalises the two-way index cut of SplitParameter to many ranges).
 *   parity   P = S_0 xor S_1 xor ... xor S_{k-1}, bit for bit (section 4.2, AEC encoding, Eq. 1;
 *            section 6: erasure coding is bitwise XOR on the parameters' bit patterns).
 *   decode   S_j = P xor (xor of all S_s, s != j)   (section 4.2, AEC decoding, Eq. 2).
 *   load     The inverse slicing of the stream back into the tensors (section 4.3, step 1).
 *
 * Every loop is over single bytes.  The only concession to speed is an optional OpenMP split of
 * the outer byte range (oracle_set_threads); the arithmetic per byte is unchanged.
 *
 * Return value of every function: 0 on success, -1 on an invalid argument.
 */
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int g_threads = 1;

void oracle_set_threads(int n) { g_threads = n < 1 ? 1 : n; }

int oracle_get_threads(void) { return g_threads; }

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Sum of the span sizes = length L of the stream. */
uint64_t oracle_stream_bytes(const uint64_t *span_nbytes, uint64_t T)
{
    uint64_t L = 0;
    for (uint64_t t = 0; t < T; ++t) L += span_nbytes[t];
    return L;
}

/* stream = span_0 || span_1 || ... || span_{T-1}.  Zero-length spans contribute nothing. */
int oracle_pack(const uint8_t *const *spans, const uint64_t *span_nbytes, uint64_t T,
                uint8_t *stream, uint64_t stream_cap)
{
    if (oracle_stream_bytes(span_nbytes, T) > stream_cap) return -1;
    uint64_t o = 0;
    for (uint64_t t = 0; t < T; ++t) {
        const uint8_t *src = spans[t];
        const uint64_t n = span_nbytes[t];
#pragma omp parallel for num_threads(g_threads) schedule(static) if (n > (1u << 20))
        for (uint64_t i = 0; i < n; ++i) stream[o + i] = src[i];
        o += n;
    }
    return 0;
}

/*
 * The bucketed snapshot, step by step: for each bucket b in turn, for each stream offset o in
 * [B_b, B_{b+1}), find the span that owns offset o and copy that one byte to host[o].
 * Buckets must have positive length and together cover exactly [0, L).
 */
int oracle_pack_bucketed(const uint8_t *const *spans, const uint64_t *span_nbytes, uint64_t T,
                         const uint64_t *bucket_nbytes, uint64_t NB,
                         uint8_t *host, uint64_t host_cap)
{
    const uint64_t L = oracle_stream_bytes(span_nbytes, T);
    if (L > host_cap) return -1;
    uint64_t covered = 0;
    for (uint64_t b = 0; b < NB; ++b) {
        if (bucket_nbytes[b] == 0) return -1;
        covered += bucket_nbytes[b];
    }
    if (covered != L) return -1;

    uint64_t B = 0;                 /* start of the current bucket in the stream */
    for (uint64_t b = 0; b < NB; ++b) {
        const uint64_t E = B + bucket_nbytes[b];
        /* locate the span that owns offset B */
        uint64_t t = 0, span_start = 0;
        while (t < T && span_start + span_nbytes[t] <= B) { span_start += span_nbytes[t]; ++t; }
        for (uint64_t o = B; o < E; ++o) {
            while (o >= span_start + span_nbytes[t]) { span_start += span_nbytes[t]; ++t; }
            host[o] = spans[t][o - span_start];
        }
        B = E;
    }
    return 0;
}

/* Inverse of oracle_pack: span_t = stream[off_t : off_t + nbytes_t]. */
int oracle_unpack(const uint8_t *stream, uint64_t stream_bytes,
                  const uint64_t *span_nbytes, uint64_t T, uint8_t *const *spans_out)
{
    if (oracle_stream_bytes(span_nbytes, T) != stream_bytes) return -1;
    uint64_t o = 0;
    for (uint64_t t = 0; t < T; ++t) {
        uint8_t *dst = spans_out[t];
        const uint64_t n = span_nbytes[t];
#pragma omp parallel for num_threads(g_threads) schedule(static) if (n > (1u << 20))
        for (uint64_t i = 0; i < n; ++i) dst[i] = stream[o + i];
        o += n;
    }
    return 0;
}

/* parity[i] = shards[0][i] ^ ... ^ shards[k-1][i], i in [0, L).  k >= 1. */
int oracle_encode(const uint8_t *const *shards, uint32_t k, uint64_t L, uint8_t *parity)
{
    if (k < 1) return -1;
#pragma omp parallel for num_threads(g_threads) schedule(static) if (L > (1u << 20))
    for (uint64_t i = 0; i < L; ++i) {
        uint8_t p = 0;
        for (uint32_t s = 0; s < k; ++s) p ^= shards[s][i];
        parity[i] = p;
    }
    return 0;
}

/*
 * Shards of unequal length: each is taken as zero-extended to Lmax = max length (0 is the
 * identity of XOR).  Not reachable through the GPU library (it rejects unequal lengths); kept to
 * state the reading and for a unit test.
 */
int oracle_encode_padded(const uint8_t *const *shards, const uint64_t *lens, uint32_t k,
                         uint8_t *parity, uint64_t parity_cap)
{
    if (k < 1) return -1;
    uint64_t Lmax = 0;
    for (uint32_t s = 0; s < k; ++s) if (lens[s] > Lmax) Lmax = lens[s];
    if (Lmax > parity_cap) return -1;
    for (uint64_t i = 0; i < Lmax; ++i) {
        uint8_t p = 0;
        for (uint32_t s = 0; s < k; ++s) p ^= (i < lens[s]) ? shards[s][i] : 0;
        parity[i] = p;
    }
    return 0;
}

/* out[i] = parity[i] ^ survivors[0][i] ^ ... ^ survivors[n-1][i]; n = k-1 may be 0. */
int oracle_reconstruct(const uint8_t *const *survivors, uint32_t n_survivors,
                       const uint8_t *parity, uint64_t L, uint8_t *out)
{
#pragma omp parallel for num_threads(g_threads) schedule(static) if (L > (1u << 20))
    for (uint64_t i = 0; i < L; ++i) {
        uint8_t v = parity[i];
        for (uint32_t s = 0; s < n_survivors; ++s) v ^= survivors[s][i];
        out[i] = v;
    }
    return 0;
}

/*
 * Rotated placement of the parity (section 4.2, AEC): with m = k members in a sharding group,
 * each member's shard is cut into k-1 segments and each member stores the parity of ONE segment
 * of every OTHER member, so that every segment of every shard is protected exactly once and the
 * redundancy per member is its shard size / (k-1) (the paper's W_n / (m (m-1)) with W_n / m the
 * shard).  Eq. 1 gives the first member's unit: p_bcd0 = b_0 xor c_0 xor d_0.
 *
 * Reading taken for the general member i (the figure that shows it is not available): member i
 * protects, from shard j != i, the segment with index r(i, j) = i if i < j, else i - 1.  For i = 0
 * this is Eq. 1 literally (segment 0 of every other member); for a fixed j the indices r(i, j),
 * i != j, are 0 .. k-2, each once.
 *
 * Segments have Lseg = ceil(L / (k-1)) bytes; the last one is zero-extended (0 is the identity of
 * XOR).  k >= 2.  parity has Lseg bytes.
 */
uint64_t oracle_segment_bytes(uint64_t L, uint32_t k)
{
    return k < 2 ? 0 : (L + (k - 2)) / (k - 1);
}

static uint32_t oracle_rot_index(uint32_t i, uint32_t j) { return i < j ? i : i - 1; }

int oracle_encode_rotated(const uint8_t *const *shards, uint32_t k, uint64_t L, uint32_t member,
                          uint8_t *parity)
{
    if (k < 2 || member >= k) return -1;
    const uint64_t Lseg = oracle_segment_bytes(L, k);
    for (uint64_t x = 0; x < Lseg; ++x) {
        uint8_t p = 0;
        for (uint32_t j = 0; j < k; ++j) {
            if (j == member) continue;
            const uint64_t y = (uint64_t)oracle_rot_index(member, j) * Lseg + x;
            if (y < L) p ^= shards[j][y];
        }
        parity[x] = p;
    }
    return 0;
}

/*
 * Decode of a lost member (Eq. 2, the subtraction decoder, applied segment by segment): segment r
 * of the lost shard is protected by the member i with r(i, lost) = r; it equals that member's
 * parity unit xor the segments the unit also covers.  shards[lost] and parities[lost] are not
 * read (they were on the lost node).  out has L bytes.
 */
int oracle_reconstruct_rotated(const uint8_t *const *shards, const uint8_t *const *parities,
                               uint32_t k, uint64_t L, uint32_t lost, uint8_t *out)
{
    if (k < 2 || lost >= k) return -1;
    const uint64_t Lseg = oracle_segment_bytes(L, k);
    for (uint32_t r = 0; r + 1 < k; ++r) {
        const uint32_t i = r < lost ? r : r + 1;         /* the member with r(i, lost) == r */
        for (uint64_t x = 0; x < Lseg; ++x) {
            const uint64_t o = (uint64_t)r * Lseg + x;
            if (o >= L) break;
            uint8_t v = parities[i][x];
            for (uint32_t j = 0; j < k; ++j) {
                if (j == i || j == lost) continue;
                const uint64_t y = (uint64_t)oracle_rot_index(i, j) * Lseg + x;
                if (y < L) v ^= shards[j][y];
            }
            out[o] = v;
        }
    }
    return 0;
}


/*
 * Collaborative redundant protection (section 4.2, last paragraph): several redundancy
 * strategies enabled at once, or one strategy several times with different parameters, so that
 * several members of a sharding group may fail.  What member i of a group of k keeps in its host
 * memory, and loses with it:
 *   - its own shard S_i;
 *   - per enabled redundant copy (ARC) with offset d, 1 <= d < k: a duplicate of the shard of
 *     member (i + d) mod k ("saves shards from peer members");
 *   - if erasure coding (AEC) is enabled: its rotated parity unit U_i (oracle_encode_rotated).
 * Recovery of the lost members' shards, in the order of the loading procedure (section 4.3: take
 * what exists as a copy, decode the rest):
 *   1. a lost shard S_x whose duplicate survives - on member (x - d) mod k for some enabled
 *      offset d - is that duplicate;
 *   2. what is still missing is decoded segment by segment with the subtraction decoder (Eq. 2):
 *      segment r of S_x is covered by the unit of member i with r(i, x) = r; it can be decoded if
 *      member i survives and every other segment that unit covers is known (its shard survived,
 *      was copied in step 1, or the segment was decoded before); repeated until nothing changes.
 * The paper states the tolerance ("N or fewer failures") without a procedure; which pairs of
 * losses a given combination really survives is exactly what this function computes.
 *
 * shards[k]        surviving members' shards (entries of lost members are not read)
 * dups[n_arc * k]  dups[a * k + i] = member i's duplicate under offset arc_offsets[a] (entries of
 *                  lost members are not read)
 * units[k]         the rotated parity units, or NULL if erasure coding is not enabled (entries
 *                  of lost members are not read)
 * lost[k]          1 = member lost
 * out[k]           out[x] (L bytes) receives the recovered shard of lost member x; bytes of
 *                  segments that cannot be recovered are left untouched
 * seg_known[k * (k-1)]  receives 1 for every segment of every member's shard that is known at
 *                  the end (all 1 for survivors)
 * Returns the number of segments with stream bytes that stay unknown (0 = everything recovered),
 * or -1 on an invalid argument.  k >= 2.
 */
int oracle_collab_recover(const uint8_t *const *shards, const uint8_t *const *dups,
                          const uint32_t *arc_offsets, uint32_t n_arc,
                          const uint8_t *const *units, uint32_t k, uint64_t L,
                          const uint8_t *lost, uint8_t *const *out, uint8_t *seg_known)
{
    if (k < 2) return -1;
    for (uint32_t a = 0; a < n_arc; ++a)
        if (arc_offsets[a] < 1 || arc_offsets[a] >= k) return -1;
    const uint32_t nseg = k - 1;
    const uint64_t Lseg = oracle_segment_bytes(L, k);
    for (uint32_t x = 0; x < k; ++x)
        for (uint32_t r = 0; r < nseg; ++r) seg_known[x * nseg + r] = lost[x] ? 0 : 1;

    /* step 1: redundant copies */
    for (uint32_t x = 0; x < k; ++x) {
        if (!lost[x] || seg_known[x * nseg]) continue;
        for (uint32_t a = 0; a < n_arc; ++a) {
            const uint32_t holder = (x + k - arc_offsets[a]) % k;   /* (holder + d) mod k == x */
            if (lost[holder]) continue;
            for (uint64_t o = 0; o < L; ++o) out[x][o] = dups[a * k + holder][o];
            for (uint32_t r = 0; r < nseg; ++r) seg_known[x * nseg + r] = 1;
            break;
        }
    }

    /* step 2: erasure decoding, segment by segment, until nothing changes */
    int progress = units != 0;
    while (progress) {
        progress = 0;
        for (uint32_t x = 0; x < k; ++x) {
            if (!lost[x]) continue;
            for (uint32_t r = 0; r < nseg; ++r) {
                if (seg_known[x * nseg + r]) continue;
                const uint32_t i = r < x ? r : r + 1;               /* r(i, x) == r */
                if (lost[i]) continue;
                int ready = 1;
                for (uint32_t j = 0; j < k; ++j)
                    if (j != i && j != x && !seg_known[j * nseg + oracle_rot_index(i, j)]) ready = 0;
                if (!ready) continue;
                for (uint64_t t = 0; t < Lseg; ++t) {
                    const uint64_t o = (uint64_t)r * Lseg + t;
                    if (o >= L) break;
                    uint8_t v = units[i][t];
                    for (uint32_t j = 0; j < k; ++j) {
                        if (j == i || j == x) continue;
                        const uint64_t y = (uint64_t)oracle_rot_index(i, j) * Lseg + t;
                        if (y < L) v ^= lost[j] ? out[j][y] : shards[j][y];
                    }
                    out[x][o] = v;
                }
                seg_known[x * nseg + r] = 1;
                progress = 1;
            }
        }
    }

    int unknown = 0;
    for (uint32_t x = 0; x < k; ++x)
        for (uint32_t r = 0; r < nseg; ++r)
            if (!seg_known[x * nseg + r] && (uint64_t)r * Lseg < L) ++unknown;
    return unknown;
}
