// Internal interface between the C-ABI host logic (reft_api.hip) and the kernels
// (reft_kernels.hip).  Not installed; the public boundary is include/reft.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace reft {

constexpr int kThreads = 256;      // 4 wavefronts of 64 lanes per workgroup
constexpr int kMaxSrc = 8;         // sources XORed by one launch; more are chained

struct LaunchCfg {
    uint32_t max_wgs;              // cap on the grid size (>= 1)
    uint32_t unroll;               // 1, 2 or 4 chunks of 16 B in flight per thread and source
    bool nontemporal;
    uint32_t small_pieces;         // a tile in which at least this many spans start takes the
                                   // LDS-staged small-piece path (0xffffffff = never)
};

// Device-side tables of a plan.
struct PlanTables {
    const uint64_t *off;           // [T+1] prefix sums of the span sizes (stream offsets)
    const uint32_t *first_span;    // [ntiles] first span that owns a byte of tile t
    uint64_t T;
    uint64_t L;
    uint32_t tile_shift;           // tile = 1 << tile_shift stream bytes
};

// Parameters of the gather variant that writes in chip-wide bursts (see k_gather_burst).
struct BurstCfg {
    uint32_t *ctr;                 // 9 * 64 words of device memory for this launch alone
    uint32_t stage_bytes;          // stream bytes a workgroup buffers in LDS per round (x2 halves)
    uint32_t wgs_per_cu;           // cap on resident workgroups per compute unit
    uint32_t num_cus;
    uint32_t max_polls;            // bound on a writer wave's wait per round (0 = never wait)
    uint32_t nap;                  // pause between polls, in units of 1024 cycles
};
constexpr size_t kBurstCtrBytes = 9 * 64 * sizeof(uint32_t);
// Words kBurstDiagWord .. +2 of a counter block (a cache line of their own, behind the polled
// counter) receive the launch's diagnostics: writer-wave rounds that met, timed out, did not wait.
constexpr uint32_t kBurstDiagWord = 8 * 64 + 32;

// Sources passed by value for the contiguous XOR kernel.
struct SrcBases {
    uint64_t p[kMaxSrc];
};

// The destination address of stream byte o, for o in [lo, hi), is dst_vbase + o, or, when dtab
// (one row of T span pointers) is not null, the byte's place in the destination's own span.
// tab holds nrows rows of T span pointers (row stride T); the kernel XORs the rows' streams and,
// if acc, the destination's current contents.  nrows + acc <= kMaxSrc.
hipError_t launch_gather(const PlanTables &pt, const uint64_t *tab, int nrows, bool acc,
                         const uint64_t *dtab, uint64_t dst_vbase, uint64_t lo, uint64_t hi,
                         const LaunchCfg &cfg, hipStream_t stream);

// The same result as launch_gather, by the burst kernel.  With dtab == null the destination is
// contiguous and vb its virtual base.  With dtab, every span with bytes must
// satisfy (dtab[i] - off[i]) mod 16 == vb mod 16 (the caller checks; otherwise use launch_gather).
// stage_bytes: a multiple of 4096, at most 65536.
hipError_t launch_gather_burst(const PlanTables &pt, const uint64_t *tab, int nrows, bool acc,
                               const uint64_t *dtab, uint64_t vb, uint64_t lo, uint64_t hi,
                               const LaunchCfg &cfg, const BurstCfg &bc, hipStream_t stream);

// Fused pack + encode: the parity of the nrows rows (contiguous, virtual base vb) and, in the same
// pass, the packed stream of row 0 (contiguous, virtual base vb2, congruent to vb modulo 16).
// The kernel keeps two LDS images per half: 4 * (stage_bytes + 16) bytes per workgroup.
hipError_t launch_gather_burst_pack(const PlanTables &pt, const uint64_t *tab, int nrows, uint64_t vb,
                                    uint64_t vb2, uint64_t lo, uint64_t hi, const LaunchCfg &cfg,
                                    const BurstCfg &bc, hipStream_t stream);

// src_vbase + o is the source address of stream byte o; tab is one row of T span pointers.
hipError_t launch_scatter(const PlanTables &pt, const uint64_t *tab, uint64_t src_vbase,
                          uint64_t lo, uint64_t hi, const LaunchCfg &cfg, hipStream_t stream);

// dst[i] = XOR over s < nsrc of src.p[s][i], i in [0, L); any alignment.  The _burst form gives the
// same bytes with reads and writes separated in time (see k_gather_burst).
hipError_t launch_xor_contig(const SrcBases &src, int nsrc, uint64_t dst, uint64_t L,
                             uint32_t tile_shift, const LaunchCfg &cfg, hipStream_t stream);
hipError_t launch_xor_contig_burst(const SrcBases &src, int nsrc, uint64_t dst, uint64_t L,
                                   const LaunchCfg &cfg, const BurstCfg &bc, hipStream_t stream);

}  // namespace reft
