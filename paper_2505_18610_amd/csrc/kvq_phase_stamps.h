// Measurement aid, not part of the library proper: in a build with -DKVQ_PHASE_STAMPS the attention kernels record
// the device wall clock (100 MHz) when thread 0 of a workgroup passes a numbered point, into a static device array
// that kvq_phase_stamps_read copies out.  paper_2505_18610_amd/phase_table.py turns the stamps of launches inside
// back-to-back trains into the per-phase table kept under profiles/.  The stamps cost about 1.5 us per launch.
//   0 workgroup entry          1 q and page descriptors staged     2 thread 0's wavefront has finished its range
//   6 all eight wavefronts joined                                   3 wavefront partials merged (LDS)
//   4 partial published and arrival ticket drawn                    5 split partials merged (last workgroup of a unit)
//   7 hardware ids: XCC_ID << 32 | HW_ID
#ifndef KVQ_PHASE_STAMPS_H
#define KVQ_PHASE_STAMPS_H

#define KVQ_STAMP_WGS 1024
#define KVQ_STAMP_SLOTS 8
static __device__ unsigned long long kvq_phase_stamps[KVQ_STAMP_WGS * KVQ_STAMP_SLOTS];
#define KVQ_STAMP_AT(k) kvq_phase_stamps[(blockIdx.y * gridDim.x + blockIdx.x) % KVQ_STAMP_WGS * KVQ_STAMP_SLOTS + (k)]
#define KVQ_STAMP(k) do { if (threadIdx.x == 0) KVQ_STAMP_AT(k) = wall_clock64(); } while (0)
#define KVQ_STAMP_ID() do { if (threadIdx.x == 0) KVQ_STAMP_AT(7) = ((unsigned long long)__builtin_amdgcn_s_getreg(20 | (31 << 11)) << 32) | (unsigned)__builtin_amdgcn_s_getreg(4 | (31 << 11)); } while (0)

#endif
