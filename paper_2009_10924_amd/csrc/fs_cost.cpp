#include "fs_cost.hpp"

#include <algorithm>
#include <cmath>

namespace fs {

const DeviceModel& device() {
  static const DeviceModel d;
  return d;
}

CostResult evaluate(const KernelCost& k, int32_t vgprs_compiled) {
  const DeviceModel& d = device();
  CostResult r;
  r.vgprs = vgprs_compiled > 0 ? vgprs_compiled : k.vgpr_estimate;

  // Occupancy from registers, LDS and workgroup shape (Section 4.3).
  const uint32_t vg = std::max<uint32_t>(d.vgpr_granule, (r.vgprs + d.vgpr_granule - 1) / d.vgpr_granule * d.vgpr_granule);
  uint32_t occ = std::min<uint32_t>(d.max_waves_per_simd, d.vgpr_per_simd_lane / vg);
  const uint32_t wpb = std::max(1, k.waves_per_block);
  uint32_t blocks_per_cu = occ * d.simd_per_cu / wpb;
  if (k.lds_bytes_per_block > 0) blocks_per_cu = std::min<uint32_t>(blocks_per_cu, d.lds_per_cu / (uint32_t)k.lds_bytes_per_block);
  blocks_per_cu = std::max<uint32_t>(1, blocks_per_cu);
  const double waves_per_cu = std::min<double>(occ * d.simd_per_cu, (double)blocks_per_cu * wpb);
  r.waves_per_simd = (int32_t)std::max(1.0, std::floor(waves_per_cu / d.simd_per_cu));

  // N_wave: rounds of resident wavefronts.
  const double capacity = waves_per_cu * d.n_cu;
  const double resident = std::min(k.waves, capacity);
  const double rounds_exact = std::max(1.0, k.waves / capacity);
  const double rounds = std::ceil(rounds_exact - 1e-9);

  // L_warp: one trip of a wave = dependent memory phases + its instruction stream while
  // sharing the SIMD with the other resident waves.
  const double util = std::max(0.05, k.lane_utilisation);
  const double elems_per_wave_trip = k.elems / std::max(1.0, k.waves * k.rows_per_wave_loop);
  const double wave_instr = elems_per_wave_trip / 64.0 / util;
  const double cycles = wave_instr * (k.valu_per_elem * d.cycles_valu + k.trans_per_elem * d.cycles_trans) +
                        k.xlane_steps * d.cycles_xlane;
  const double simd_share = std::max(1.0, resident / (d.n_cu * d.simd_per_cu));
  // two or three waves on a SIMD do not cover each other's instruction latencies (dependent transcendental chains show:
  // measured 4 % on rows kept in registers at two waves against four)
  const double issue_stall = r.waves_per_simd < 4 ? 1.0 + 0.025 * (4 - r.waves_per_simd) : 1.0;
  const double t_issue = cycles * simd_share * issue_stall / d.clock_hz;
  const double t_trip = k.dep_phases * d.mem_latency_s + k.barriers * d.barrier_s + t_issue;
  const double t_latency = rounds * k.rows_per_wave_loop * t_trip;

  // Streaming floor.  Achievable bandwidth = the measured copy rate, derated for
  //   * bytes in flight (Little's law),
  //   * short contiguous runs per access (a row group of L lanes touches L*16 bytes),
  //   * lanes that hold padding (their clamped loads still occupy the memory pipeline),
  //   * a last, partly filled round of wavefronts.
  const double in_flight = resident * 64.0 * k.bytes_in_flight_per_lane * util;
  double bw = std::min(d.hbm_peak_Bps * d.stream_fraction, in_flight / d.mem_latency_s);
  if (k.access_run_bytes > 0 && k.access_run_bytes < 128) bw /= 1.0 + 0.2 * (128.0 / k.access_run_bytes - 1.0);
  if (k.store_run_bytes > 0 && k.store_run_bytes < 512) bw *= 0.97;
  bw /= 1.0 + 0.3 * (1.0 / util - 1.0);
  bw /= 1.0 + 0.25 * (rounds / rounds_exact - 1.0);
  if (occ < 4) bw /= 1.0 + 0.04 * (4.0 - occ);   // few waves per SIMD: a wave's own stalls are not covered
  const double t_hbm = k.hbm_bytes / bw;
  const double t_cache = k.cache_bytes / d.l2_Bps;
  const double t_lds = k.lds_traffic_bytes / d.lds_Bps;
  const double t_alu = k.elems / util / 64.0 * (k.valu_per_elem * d.cycles_valu + k.trans_per_elem * d.cycles_trans) /
                       (d.n_cu * d.simd_per_cu) / d.clock_hz;
  // every extra round of a kernel that runs in few rounds pays a ramp of its own;
  // so does a wave that has to wait for its index arithmetic before its first load
  const double t_ramp = std::min(rounds - 1.0, 2.0) * 0.25 * d.mem_latency_s +
                        k.preamble_instr * d.cycles_valu * simd_share / d.clock_hz;

  // The wave-rounds term and the streaming floor overlap only partly: a wave that is
  // computing is not loading, and only the other waves of its SIMD can fill the gap.
  // (re-reads that the caches serve share the memory pipeline with the stream but mostly fill its gaps: a quarter
  // of their own time shows, measured on the patterns with per-column operands)
  const double t_stream = std::max(t_hbm + 0.25 * t_cache + t_lds, t_alu);
  const double t_body = std::max(t_latency, t_stream) + 0.10 * std::min(t_latency, t_stream);
  r.seconds = d.launch_s + t_body + t_ramp + k.serial_tail_s;
  return r;
}

}  // namespace fs
