"""The public header must be plain C (callers may not be C++), and the oracle must be clean
under the address and undefined-behaviour sanitizers (host code only; CPU tests)."""
import os
import subprocess
import sys
import textwrap

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_compiles_as_c99(tmp_path):
    src = tmp_path / "use_evg.c"
    src.write_text(textwrap.dedent("""
        #include "evg.h"
        #include <stddef.h>
        int main(void) {
          evg_config cfg;
          evg_stats_t st;
          evg_ctx* ctx = NULL;
          double ms[EVG_PH_COUNT];
          uint64_t n[EVG_PH_COUNT];
          (void)cfg; (void)st; (void)ms; (void)n;
          /* every entry point must be declared with a C prototype */
          (void)evg_padded_numel; (void)evg_layer_offsets; (void)evg_init; (void)evg_step;
          (void)evg_stats; (void)evg_last_decisions; (void)evg_message; (void)evg_average;
          (void)evg_state_size; (void)evg_state_export; (void)evg_state_import;
          (void)evg_timing; (void)evg_timing_read; (void)evg_destroy; (void)evg_strerror;
          (void)evg_error_text; (void)evg_step_next; (void)evg_message_hashes;
          return ctx != NULL;
        }
    """))
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic",
                    "-I", os.path.join(ROOT, "include"), "-c", str(src), "-o", str(tmp_path / "use_evg.o")],
                   check=True)


DRIVER = r"""
#include <cstdint>
#include <cstdio>
#include <vector>
extern "C" {
struct orc_config { uint32_t P, L; const uint64_t* layer_numel; const uint32_t* layer_fan_in; float lr, momentum;
  uint32_t thr_mode; float thr_fixed; float horizon; uint32_t hist_len; float delta_init; uint32_t force_first;
  uint32_t topk_ppm, topk_key, trigger_kind, grad_mode; uint64_t seed; uint32_t dist, fan_in_scaling;
  double sigma0, decay; float spike_prob, spike_gain; uint32_t delivery_delay, xhat_reset; };
void* orc_create(const orc_config*, const float*);
int orc_step(void*, uint64_t, const float*, const int8_t*);
void orc_totals(void*, uint64_t*);
void orc_destroy(void*);
}
int main() {
  const uint64_t numel[4] = {4097, 1, 130, 7};
  const uint32_t fan[4] = {16, 16, 8, 8};
  uint64_t N = 0; for (uint64_t n : numel) N += n;
  uint64_t events = 0;
  for (int mode = 0; mode < 7; ++mode) {
    orc_config c{};
    c.P = 4; c.L = 4; c.layer_numel = numel; c.layer_fan_in = fan; c.lr = 0.05f; c.momentum = 0.9f;
    c.thr_mode = 1; c.horizon = 1.0f; c.hist_len = mode == 1 ? 3 : 1; c.force_first = 1;
    c.topk_ppm = mode >= 2 ? 100000 : 0; c.topk_key = mode == 3; c.trigger_kind = mode == 4;
    c.delivery_delay = mode == 5; c.xhat_reset = mode == 6; c.seed = 99; c.dist = mode == 2; c.fan_in_scaling = 1;
    c.sigma0 = 0.05; c.decay = 0.98; c.spike_prob = 0.2f; c.spike_gain = 5.0f;
    std::vector<float> x0(c.P * N, 0.25f);
    void* h = orc_create(&c, x0.data());
    if (!h) return 2;
    for (uint64_t k = 0; k < 25; ++k) if (orc_step(h, k, nullptr, nullptr)) return 3;
    uint64_t t[8]; orc_totals(h, t); events += t[0];
    orc_destroy(h);
  }
  std::printf("events %llu\n", (unsigned long long)events);
  return events > 0 ? 0 : 4;
}
"""


def test_oracle_is_clean_under_sanitizers(tmp_path):
    drv = tmp_path / "drive.cpp"
    drv.write_text(DRIVER)
    exe = tmp_path / "drive"
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-ffp-contract=off", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan", str(drv), os.path.join(ROOT, "oracle", "evg_oracle.cpp"),
                    "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    sys.stdout.write(out.stdout + out.stderr)
    assert out.returncode == 0, out.stderr
