// Latency evaluator for one kernel launch, in the shape of the paper's Eq. 1
// (L = N_wave x L_warp, N_wave = N_warp / Occupancy, L_warp = N_instruction x CPI),
// re-derived for a bandwidth-bound part: the wave-rounds term is kept, and a
// streaming floor (bytes / achievable HBM bandwidth) is added because on MI355X these
// kernels run at the memory roofline, not at the instruction-issue limit.
#pragma once
#include <cstdint>

namespace fs {

struct DeviceModel {
  // MI355X (gfx950) public figures
  uint32_t n_cu = 256;
  uint32_t simd_per_cu = 4;
  uint32_t max_waves_per_simd = 8;
  uint32_t vgpr_per_simd_lane = 512;
  uint32_t vgpr_granule = 8;
  uint32_t lds_per_cu = 160 * 1024;
  double clock_hz = 2.4e9;
  double hbm_peak_Bps = 8.0e12;
  // measured / calibrated on one MI355X
  double stream_fraction = 0.84;     // one-shot kernels with three or more independent streams, fraction of hbm_peak
                                     // (the grid-stride copy kernel reaches 0.78)
  double mem_latency_s = 1.2e-6;     // loaded HBM round trip seen by a wave
  double launch_s = 2.2e-6;          // fixed cost of one kernel: dispatch, first load round trip, drain
  double l2_Bps = 20.0e12;           // aggregate cache bandwidth for re-read operands
  double last_level_cache_bytes = 256.0 * 1024 * 1024;   // memory-side cache in front of HBM
  double last_level_reread = 0.45;   // time of a re-read that the memory-side cache still holds, relative to HBM (measured)
  double lds_Bps = 60.0e12;          // aggregate LDS bandwidth
  double barrier_s = 0.15e-6;        // one workgroup barrier incl. the LDS round trip
  double cycles_valu = 4.0;          // issue cycles of one wave-wide VALU op on a 16-lane SIMD
  double cycles_trans = 16.0;        // quarter-rate transcendental
  double cycles_xlane = 12.0;        // DPP / permute step incl. its dependency stall
};
const DeviceModel& device();

// What one candidate kernel does, as the enumerator describes it.
struct KernelCost {
  double hbm_bytes = 0;                 // bytes that must cross HBM
  double cache_bytes = 0;               // re-reads served by L1/L2
  double lds_traffic_bytes = 0;
  double elems = 0;
  double valu_per_elem = 0;             // plain VALU ops per element
  double trans_per_elem = 0;            // quarter-rate ops per element
  double waves = 0;                     // wavefronts launched
  int32_t waves_per_block = 4;
  double bytes_in_flight_per_lane = 16; // independent load bytes a lane has outstanding
  double rows_per_wave_loop = 1;        // sequential trips of the kernel's outer loop per wave
  int32_t dep_phases = 1;               // dependent global-memory phases per trip
  int32_t xlane_steps = 0;              // cross-lane steps per trip
  int32_t barriers = 0;                 // workgroup barriers per trip
  int32_t vgpr_estimate = 32;
  int32_t lds_bytes_per_block = 0;
  double lane_utilisation = 1.0;        // fraction of lanes holding data
  double access_run_bytes = 0;          // contiguous bytes one row group touches per load (0 = long)
  double store_run_bytes = 0;           // contiguous run written by one store instruction group (0 = long)
  double preamble_instr = 40;           // VALU instructions a wave runs before it can issue its first load
  double serial_tail_s = 0;             // work done by a single workgroup after the rest finished
};

struct CostResult {
  double seconds = 0;
  int32_t waves_per_simd = 0;
  int32_t vgprs = 0;
};
CostResult evaluate(const KernelCost& k, int32_t vgprs_compiled);

}  // namespace fs
